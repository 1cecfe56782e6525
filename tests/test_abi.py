"""CPU-side checks of the C ABI: the library loads, exports every declared symbol and rejects bad
arguments on the host before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2408_00264_amd import clover, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(clover.LIB_PATH):
        from paper_2408_00264_amd import build
        build.build()
    return clover.load_library()


def test_header_symbols_exported(lib):
    text = open(os.path.join(ROOT, "include", "clover.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b([a-z_][a-z0-9_]*)\s*\(", text))
    names -= {"defined"}
    declared = {n for n in names if n.startswith("clover_") or
                n in ("draft_tree", "verify_tree", "accept_and_compact", "accept_and_compact_sampled")}
    assert {"clover_init", "draft_tree", "verify_tree", "accept_and_compact"} <= declared
    for n in declared:
        assert hasattr(lib, n), n
    assert declared == set(clover.EXPORTS)


def test_struct_layout_matches_header():
    assert C.sizeof(clover.Config) == 18 * 4
    assert C.sizeof(clover.LayerWeights) == 9 * 8
    assert C.sizeof(clover.ADWeights) == 7 * 8
    assert C.sizeof(clover.Weights) == 8 * (4 + 7 + 7 + 1 + 2 + 2 + 1)


def _cfg(**kw):
    shape = synth.scaled(synth.CONFIGS[1], **{k: v for k, v in kw.items() if hasattr(synth.CONFIGS[1], k)})
    c = clover.make_config(shape, kw.get("max_batch", 1), kw.get("max_seq", 128), kw.get("max_nodes", 16))
    return c


def test_workspace_bytes_and_config_errors(lib):
    n = C.c_size_t()
    assert lib.clover_workspace_bytes(C.byref(_cfg()), C.byref(n)) == 0 and n.value > 0
    small = n.value
    assert lib.clover_workspace_bytes(C.byref(_cfg(max_seq=1024)), C.byref(n)) == 0 and n.value > small
    assert lib.clover_workspace_bytes(None, C.byref(n)) == clover.E_NULL
    bad = _cfg(); bad.ad_heads = 7            # hidden 256 is not a multiple of 7 heads
    assert lib.clover_workspace_bytes(C.byref(bad), C.byref(n)) == clover.E_CONFIG
    assert b"ad_heads" in lib.clover_last_global_error()
    bad = _cfg(); bad.n_kv_heads = 3
    assert lib.clover_workspace_bytes(C.byref(bad), C.byref(n)) == clover.E_CONFIG
    bad = _cfg(); bad.max_nodes = 129
    assert lib.clover_workspace_bytes(C.byref(bad), C.byref(n)) == clover.E_CONFIG
    wide = _cfg(max_seq=512); wide.max_nodes = 200; wide.flags = clover.FLAG_INTERVAL_MASK   # the linear-size mask lifts the bound
    assert lib.clover_workspace_bytes(C.byref(wide), C.byref(n)) == 0
    wide.max_nodes = 257
    assert lib.clover_workspace_bytes(C.byref(wide), C.byref(n)) == clover.E_CONFIG
    bad = _cfg(max_seq=120)                   # the caches are pools of 32-position pages
    assert lib.clover_workspace_bytes(C.byref(bad), C.byref(n)) == clover.E_CONFIG
    bad = _cfg(); bad.dtype = 5
    assert lib.clover_workspace_bytes(C.byref(bad), C.byref(n)) == clover.E_CONFIG
    bad = _cfg(); bad.prefill_rows = 257
    assert lib.clover_workspace_bytes(C.byref(bad), C.byref(n)) == clover.E_CONFIG
    wide = _cfg(); wide.prefill_rows = 256     # row buffers sized for the prefill passes
    assert lib.clover_workspace_bytes(C.byref(wide), C.byref(n)) == 0 and n.value > small
    # LLaMA3-8B-shaped batch-1 context: the fragment-major copy of every linear weight (16.1 GB, as large as
    # the weights themselves) plus a few hundred MB of caches and activations
    big = clover.make_config(synth.CONFIGS[3], 1, 2048, 64)
    assert lib.clover_workspace_bytes(C.byref(big), C.byref(n)) == 0 and 1.6e10 < n.value < 1.8e10


def test_init_rejects_bad_arguments_on_host(lib):
    cfg = _cfg()
    ctx = C.c_void_p()
    assert lib.clover_init(C.byref(cfg), None, None, None, 0, None, C.byref(ctx)) == clover.E_NULL
    # fake, never dereferenced device pointers: validation happens before any launch
    fake = 0x1000
    L = (clover.LayerWeights * 2)(*[clover.LayerWeights(*([fake] * 9)) for _ in range(2)])
    fc = (C.c_void_p * 3)(None, fake, fake)
    ad = clover.ADWeights(*([fake] * 7))
    w = clover.Weights(fake, L, fake, fake, ad, ad, L, fake, fake, fc, fc, fake)

    def tree(parent, rank):
        p = np.asarray(parent, np.int32); r = np.asarray(rank, np.int32)
        return clover.Tree(len(p), p.ctypes.data_as(C.POINTER(C.c_int32)), r.ctypes.data_as(C.POINTER(C.c_int32))), (p, r)

    for parent, rank, why in [([0, 0], [0, 0], b"parent[0]"), ([-1, 1], [0, 0], b"parent index"),
                              ([-1, 0, 0], [0, 1, 1], b"distinct"), ([-1, 0, 0, 2, 1], [0, 0, 1, 0, 0], b"breadth-first"),
                              ([-1, 0], [0, 16], b"rank")]:
        t, keep = tree(parent, rank)
        rc = lib.clover_init(C.byref(cfg), C.byref(w), C.byref(t), C.c_void_p(0x10000), 1 << 40, None, C.byref(ctx))
        assert rc == clover.E_TREE, (parent, rc)
        assert why in lib.clover_last_global_error(), lib.clover_last_global_error()
    t, keep = tree(list(range(-1, 16)), [0] * 17)          # 17 nodes > max_nodes 16
    assert lib.clover_init(C.byref(cfg), C.byref(w), C.byref(t), C.c_void_p(0x10000), 1 << 40, None, C.byref(ctx)) == clover.E_TREE
    t, keep = tree([-1, 0], [0, 0])
    assert lib.clover_init(C.byref(cfg), C.byref(w), C.byref(t), C.c_void_p(0x10001), 1 << 40, None, C.byref(ctx)) == clover.E_CONFIG
    w2 = clover.Weights(fake, L, fake, None, ad, ad, L, fake, fake, fc, fc, fake)
    assert lib.clover_init(C.byref(cfg), C.byref(w2), C.byref(t), C.c_void_p(0x10000), 1 << 40, None, C.byref(ctx)) == clover.E_NULL


def test_null_context_calls(lib):
    assert lib.draft_tree(None, 1, None, None, None, None) == clover.E_NULL
    assert lib.verify_tree(None, 1, None, None, None) == clover.E_NULL
    assert lib.accept_and_compact(None, 1, None, None, None, None, None, None, None, None) == clover.E_NULL
    assert lib.clover_destroy(None) == clover.E_NULL
    assert lib.clover_kernel_class_count() >= 10
    assert lib.clover_kernel_class_name(0) == b"embed"
    assert lib.clover_op_gemm(0, 0, None, None, None, 4, 1, 4, 4, None, 0, None) == clover.E_NULL


def test_shipped_library_reads_no_environment_switch(lib):
    """The library's behaviour must not depend on the environment: the shipped build neither imports getenv nor
    carries the name of a CLOVER_* switch (those exist only in -DCLOVER_ABLATE tuning builds)."""
    assert b"CLOVER_NO_PANEL" not in open(clover.LIB_PATH, "rb").read()
    import subprocess
    blob = open(clover.LIB_PATH, "rb").read()
    header = open(os.path.join(ROOT, "include", "clover.h")).read()
    for name in set(re.findall(rb"CLOVER_[A-Z0-9_]+", blob)):       # only names the header declares (error messages)
        assert name.decode() in header, name
    syms = subprocess.run(["nm", "-D", clover.LIB_PATH], capture_output=True, text=True).stdout
    assert "getenv" not in syms


def test_tuning_builds_never_overwrite_the_shipped_library():
    """Ablation switches and extra macros exist only in builds that name their own output file."""
    from paper_2408_00264_amd import build as B
    with pytest.raises(ValueError):
        B.build(ablate=True)                                   # no output path
    with pytest.raises(ValueError):
        B.build(defines=("CLOVER_TILE_ABLATE=1",), out="/tmp/x.so")   # macros without --ablate
    with pytest.raises(ValueError):
        B.build(ablate=True, defines=("CLOVER_TILE_ABLATE=1",))
