"""Host-side checks of the C ABI that need no GPU: exported symbols, struct layout, the host
logic (retained counts, cache-state schedule, workspace sizing) and argument rejection."""
import ctypes
import os
import re
import subprocess
import sys

import pytest

from oracle import sdllm_oracle as orc
from paper_2508_02558_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2508_02558_amd.build import build_library
        build_library(verbose=False)
    return B.load()


def _declared_functions():
    names = set()
    for header in sorted(os.listdir(INCLUDE)):
        if header.endswith(".h"):
            text = open(os.path.join(INCLUDE, header)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(sdllm_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    declared = _declared_functions()
    assert set(declared) == set(B.EXPORTED)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layout_matches_the_header(tmp_path):
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "sdllm.h"\n'
                   'int main(void){printf("%zu %zu %zu %zu %zu\\n", sizeof(sdllm_shape_t),'
                   ' offsetof(sdllm_shape_t, softmax_scale), offsetof(sdllm_shape_t, retention),'
                   ' offsetof(sdllm_shape_t, q_stride), offsetof(sdllm_shape_t, out_stride));return 0;}\n')
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    S = B.sdllm_shape_t
    assert got == [ctypes.sizeof(S), S.softmax_scale.offset, S.retention.offset, S.q_stride.offset, S.out_stride.offset]


def _shape(**kw):
    base = dict(batch=1, n_q_heads=2, n_kv_heads=2, head_dim=64, seq_len=160, block_off=64, block_len=32,
                dtype=B.SDLLM_F32, retention=0.5, pool_kernel=3)
    base.update(kw)
    return B.make_shape(**base)


def test_retained_count_agrees_with_golden_table_and_oracle(lib, golden):
    for r, n, ceil_k, floor_k in golden("retained_count_table.txt"):
        n = int(n)
        # prefix of n tokens, block right after it, no suffix
        for rounding, want in ((B.SDLLM_CEIL, int(ceil_k)), (B.SDLLM_FLOOR, int(floor_k))):
            s = _shape(seq_len=n + 32, block_off=n, retention=float(r), k_rounding=rounding)
            kt, kp, ks = B.sdllm_retained_count(s)
            assert (kt, kp, ks) == (want, want, 0)
    s = _shape()
    assert B.sdllm_retained_count(s) == (64, 32, 32)
    s = _shape(select_mode=B.SDLLM_JOINT, k_rounding=B.SDLLM_FLOOR)
    assert B.sdllm_retained_count(s) == (64, -1, -1)
    s = _shape(evict_scope=B.SDLLM_EVICT_PREFIX_ONLY)
    assert B.sdllm_retained_count(s) == (32 + 64, 32, 64)
    for r in (0.0, 0.1, 0.3, 0.7, 0.9, 1.0):
        for n in (0, 1, 7, 10, 33):
            s = _shape(seq_len=n + 32 + 5, block_off=n, retention=r)
            assert B.sdllm_retained_count(s)[1:] == (orc.retained_count(n, r), orc.retained_count(5, r))


def test_cache_state_schedule(lib, golden):
    for delay, states in golden("cache_state_table.txt"):
        for i, st in enumerate(states.split()):
            assert B.sdllm_cache_state(i, int(delay)) == int(st)
    with pytest.raises(B.SdllmError):
        B.sdllm_cache_state(-1, 1)


def test_invalid_shapes_are_rejected(lib):
    bad = [dict(batch=0), dict(n_q_heads=3), dict(block_off=140), dict(retention=1.5), dict(retention=-0.1),
           dict(pool_kernel=2), dict(pool_kernel=0), dict(dtype=7), dict(score_mode=3), dict(select_mode=2),
           dict(k_rounding=5), dict(pool_mode=2), dict(evict_scope=2), dict(q_stride=(4096, 2048, 63)),
           dict(softmax_scale=-1.0), dict(retention=float("nan"))]
    for kw in bad:
        with pytest.raises(B.SdllmError) as ei:
            B.sdllm_retained_count(_shape(**kw))
        assert ei.value.status == B.SDLLM_ERR_INVALID_ARG, kw
    for kw in (dict(head_dim=96), dict(block_len=65, seq_len=300)):
        with pytest.raises(B.SdllmError) as ei:
            B.sdllm_retained_count(_shape(**kw))
        assert ei.value.status == B.SDLLM_ERR_UNSUPPORTED, kw
    assert B.error_string(0) == "ok" and "workspace" in B.error_string(B.SDLLM_ERR_WORKSPACE)
    assert B.sdllm_version() >= 100


def test_null_pointers_and_small_workspace_are_rejected_before_any_launch(lib):
    s = _shape()
    z = ctypes.c_void_p(None)
    sp = ctypes.byref(s)
    assert lib.sdllm_score_select(sp, z, z, z, z, z, z, 0, z) == B.SDLLM_ERR_INVALID_ARG
    assert lib.sdllm_compact_kv(sp, z, z, z, z, z, z) == B.SDLLM_ERR_INVALID_ARG
    assert lib.sdllm_sparse_attn(sp, z, z, z, 4, z, z, z, z, 0, z) == B.SDLLM_ERR_INVALID_ARG
    assert lib.sdllm_block_step(sp, 0, 1, z, z, z, z, z, z, z, z, 0, z, None) == B.SDLLM_ERR_WORKSPACE
    # a fake but aligned pointer value is enough to get past the pointer checks (nothing is enqueued
    # when the workspace is too small)
    fake = ctypes.c_void_p(0x1000)
    assert lib.sdllm_score_select(sp, fake, fake, fake, z, z, fake, 16, z) == B.SDLLM_ERR_WORKSPACE
    assert lib.sdllm_score_select(sp, fake, fake, fake, z, z, ctypes.c_void_p(0x1008), 1 << 30, z) == B.SDLLM_ERR_WORKSPACE
    assert lib.sdllm_sparse_attn(sp, ctypes.c_void_p(0x1004), z, z, 0, fake, fake, fake, z, 0, z) == B.SDLLM_ERR_INVALID_ARG
    assert lib.sdllm_sparse_attn(sp, fake, z, z, -1, fake, fake, fake, z, 0, z) == B.SDLLM_ERR_INVALID_ARG


def test_noalloc_entry_rejects_requests_beyond_its_static_scratch(lib):
    # batch 8 of a 28/4-head shape with 8000 cached keys runs the shared-tile kernel with 8 key splits:
    # 1792 partial slots of 16.25 KB, far beyond the 8 MiB array.  Rejected on the host, nothing enqueued.
    s = B.make_shape(batch=8, n_q_heads=28, n_kv_heads=4, head_dim=128, seq_len=20000, block_off=12000, block_len=32,
                     dtype=B.SDLLM_BF16, cache_rows=8000)
    assert B.sdllm_workspace_bytes(s, B.SDLLM_OP_SPARSE_ATTN, 8000) > B.SDLLM_STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)
    z = ctypes.c_void_p(None)
    assert lib.sdllm_sparse_attn_noalloc(ctypes.byref(s), fake, fake, fake, 8000, fake, fake, fake, z) == B.SDLLM_ERR_STATIC_LIMIT
    assert "static scratch" in B.error_string(B.SDLLM_ERR_STATIC_LIMIT)
    assert lib.sdllm_sparse_attn_noalloc(ctypes.byref(s), fake, fake, fake, -1, fake, fake, fake, z) == B.SDLLM_ERR_INVALID_ARG


def test_static_scratch_is_visible_in_the_device_image(lib, tmp_path):
    # hipGetSymbolAddress looks the array up by name in the gfx950 code object: it has to be a GLOBAL
    # symbol there (a LOCAL one makes the runtime abort on the first sdllm_sparse_attn_noalloc call)
    obj = os.path.join(ROOT, "paper_2508_02558_amd", "_build", "api.o")
    objdump, readelf = "/opt/rocm/llvm/bin/llvm-objdump", "/opt/rocm/llvm/bin/llvm-readelf"
    if not (os.path.exists(obj) and os.path.exists(objdump) and os.path.exists(readelf)):
        pytest.skip("needs the build directory and the LLVM binutils")
    local = tmp_path / "api.o"
    local.write_bytes(open(obj, "rb").read())
    subprocess.check_call([objdump, "--offloading", str(local)], cwd=tmp_path, stdout=subprocess.DEVNULL)
    images = [f for f in os.listdir(tmp_path) if "gfx950" in f]
    assert images, os.listdir(tmp_path)
    syms = subprocess.check_output([readelf, "--dyn-syms", str(tmp_path / images[0])], text=True)
    rows = [ln.split() for ln in syms.splitlines() if ln.strip().endswith("scratch")]
    assert rows and all(r[4] == "GLOBAL" and int(r[2]) == B.SDLLM_STATIC_SCRATCH_BYTES for r in rows), syms


def test_segments_beyond_the_selection_limit_are_rejected_before_any_launch(lib):
    # a prefix of more than 1M candidates: the selection's per-chunk tables end there
    s = B.make_shape(batch=1, n_q_heads=1, n_kv_heads=1, head_dim=128, seq_len=1_200_000 + 32, block_off=1_200_000, block_len=32,
                     dtype=B.SDLLM_BF16)
    fake = ctypes.c_void_p(0x1000)
    z = ctypes.c_void_p(None)
    assert lib.sdllm_score_select(ctypes.byref(s), fake, fake, fake, z, z, fake, 1 << 40, z) == B.SDLLM_ERR_UNSUPPORTED
    ok = B.make_shape(batch=1, n_q_heads=1, n_kv_heads=1, head_dim=128, seq_len=1_000_000 + 32, block_off=1_000_000, block_len=32,
                      dtype=B.SDLLM_BF16)
    assert B.sdllm_workspace_bytes(ok, B.SDLLM_OP_SCORE_SELECT) > 3 * 4 * 1_000_000   # scores + two key buffers


def test_workspace_sizes(lib):
    s = _shape()
    for op in (B.SDLLM_OP_SCORE_SELECT, B.SDLLM_OP_COMPACT_KV, B.SDLLM_OP_SPARSE_ATTN, B.SDLLM_OP_BLOCK_STEP):
        assert B.sdllm_workspace_bytes(s, op, 64) >= 256
    # split-KV partials of the MFMA path: a batch-1 LLaDA-shaped call needs room for them
    big = B.make_shape(batch=1, n_q_heads=32, n_kv_heads=32, head_dim=128, seq_len=4352, block_off=4096,
                       block_len=32, dtype=B.SDLLM_BF16)
    kt, _, _ = B.sdllm_retained_count(big)
    assert kt == 2160
    assert B.sdllm_workspace_bytes(big, B.SDLLM_OP_SPARSE_ATTN, kt) > 32 * 32 * 128 * 4
    assert B.sdllm_workspace_bytes(big, B.SDLLM_OP_BLOCK_STEP) >= B.sdllm_workspace_bytes(big, B.SDLLM_OP_SCORE_SELECT)
    with pytest.raises(B.SdllmError):
        B.sdllm_workspace_bytes(s, 9)


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2508_02558_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith(".py"):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f
                assert "sdllm_oracle" not in text, f
    text = open(os.path.join(ROOT, "oracle", "sdllm_oracle.py")).read()
    assert "paper_2508_02558_amd" not in text and "ctypes" not in text
