"""The C-ABI library loads and exports what include/thanos.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "thanos.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(thanos_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def L():
    import paper_2504_05346_amd as t
    if not os.path.exists(t.lib_path):
        from paper_2504_05346_amd import build
        build.build()
    return t.lib()


def test_exports_every_declared_symbol(L):
    names = _declared_functions()
    assert {"thanos_hessian_accumulate", "thanos_factor", "thanos_prune_layer",
            "thanos_factor_workspace_bytes", "thanos_prune_workspace_bytes",
            "thanos_status_string"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_diagnostic_builds_export_their_entry_points(L):
    """libthanos_timeline.so is the same library with timestamps compiled in (timeline_probe.py);
    the product library must not carry its entry points."""
    here = os.path.dirname(L._name)
    T = ctypes.CDLL(os.path.join(here, "libthanos_timeline.so"))
    for n in _declared_functions() + ["thanos_timeline_select", "thanos_timeline_read",
                                      "thanos_timeline_clear"]:
        assert hasattr(T, n), n
    assert not hasattr(L, "thanos_timeline_select")
    P = ctypes.CDLL(os.path.join(here, "libthanos_probe.so"))
    assert hasattr(P, "thanos_probe_mfma_f16") and hasattr(P, "thanos_probe_copy")


def test_status_strings(L):
    import paper_2504_05346_amd as t
    seen = {t.thanos_status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert t.thanos_status_string(99) == "unknown status"


def test_host_side_argument_checks(L):
    import paper_2504_05346_amd as t
    # NULL pointers / bad sizes are rejected before any device work
    assert L.thanos_hessian_accumulate(None, 8, None, t.THANOS_F16, 4, 8, 1.0, None) == 1
    assert L.thanos_hessian_accumulate(None, 0, None, t.THANOS_F16, 4, 8, 1.0, None) == 1
    assert L.thanos_factor(None, 8, 0.01, None, None, None, 0, None, None) == 1
    o = t.PruneOpts(mode=t.THANOS_NM, sparsity=0.0, n=2, m=4, block_size=128, damping=0.01)
    assert t.thanos_prune_workspace_bytes(64, 256, o) > 64 * 128 * 4
    assert L.thanos_prune_layer(None, t.THANOS_F16, 64, 256, None, ctypes.byref(o), None, None,
                                None, None, 0, None, None) == 1
    bad = t.PruneOpts(mode=t.THANOS_NM, sparsity=0.0, n=2, m=4, block_size=126, damping=0.01)
    assert t.thanos_prune_workspace_bytes(64, 256, bad) == 0          # m does not divide B
    # large blocks (the block-size ablation of the Experiments section): up to 4096 columns and
    # 2048 unknowns per row; their tile grids live in the workspace, not in LDS
    small = t.PruneOpts(mode=t.THANOS_UNSTRUCTURED, sparsity=0.5, n=0, m=0, block_size=256,
                        damping=0.01)
    big = t.PruneOpts(mode=t.THANOS_UNSTRUCTURED, sparsity=0.5, n=0, m=0, block_size=512,
                      damping=0.01)
    assert t.thanos_prune_workspace_bytes(64, 256, big) > t.thanos_prune_workspace_bytes(64, 256, small)
    nm512 = t.PruneOpts(mode=t.THANOS_NM, sparsity=0.0, n=2, m=4, block_size=512, damping=0.01)
    assert t.thanos_prune_workspace_bytes(64, 1024, nm512) > 0
    nm4k = t.PruneOpts(mode=t.THANOS_NM, sparsity=0.0, n=2, m=4, block_size=4096, damping=0.01)
    assert t.thanos_prune_workspace_bytes(64, 8192, nm4k) > 0          # 2048 unknowns per row
    nm34 = t.PruneOpts(mode=t.THANOS_NM, sparsity=0.0, n=3, m=4, block_size=4096, damping=0.01)
    assert t.thanos_prune_workspace_bytes(64, 8192, nm34) == 0         # 3072 unknowns per row
    nm8k = t.PruneOpts(mode=t.THANOS_NM, sparsity=0.0, n=1, m=8, block_size=8192, damping=0.01)
    assert t.thanos_prune_workspace_bytes(64, 8192, nm8k) == 0         # block wider than 4096
    un4k = t.PruneOpts(mode=t.THANOS_UNSTRUCTURED, sparsity=0.5, n=0, m=0, block_size=4096,
                       damping=0.01)
    assert t.thanos_prune_workspace_bytes(64, 8192, un4k) == 0         # a row may lose all 4096
    assert t.thanos_factor_workspace_bytes(1000) >= 3 * 1024 * 1024 * 4
    p1 = t.PruneOpts(mode=t.THANOS_UNSTRUCTURED, sparsity=1.0, n=0, m=0, block_size=128,
                     damping=0.01)
    assert t.thanos_prune_workspace_bytes(64, 256, p1) == 0           # p must be < 1


def test_workspace_too_small_is_reported(L):
    """THANOS_ERR_WORKSPACE comes from host-side checks: no pointer is dereferenced before it."""
    import paper_2504_05346_amd as t
    fake = ctypes.c_void_p(4096)          # non-NULL, 256-byte aligned, never touched
    need = t.thanos_factor_workspace_bytes(256)
    assert L.thanos_factor(fake, 256, 0.01, ctypes.c_void_p(8192), fake, fake, need - 1, fake,
                           None) == 3
    assert L.thanos_factor(fake, 256, 0.01, ctypes.c_void_p(8192), fake, None, need, fake,
                           None) == 3
    o = t.PruneOpts(mode=t.THANOS_UNSTRUCTURED, sparsity=0.5, n=0, m=0, block_size=128,
                    damping=0.01)
    need = t.thanos_prune_workspace_bytes(64, 256, o)
    assert need > 0
    assert L.thanos_prune_layer(fake, t.THANOS_F16, 64, 256, fake, ctypes.byref(o), fake, None,
                                fake, fake, need - 1, fake, None) == 3
    assert t.thanos_status_string(3) == "workspace too small"
    # U must not alias H; a given mask and outlier rows exclude each other
    assert L.thanos_factor(fake, 256, 0.01, fake, fake, fake, 1 << 30, fake, None) == 1
    om = t.PruneOpts(mode=t.THANOS_NM, sparsity=0.0, n=2, m=4, block_size=128, damping=0.01,
                     outlier_fraction=0.1)
    om.mask_in = 4096
    assert L.thanos_prune_layer(fake, t.THANOS_F16, 64, 256, fake, ctypes.byref(om), fake, None,
                                fake, fake, 1 << 30, fake, None) == 2
    # the structured mode puts rows in grid.y
    so = t.PruneOpts(mode=t.THANOS_STRUCTURED, sparsity=0.3, n=0, m=0, block_size=128,
                     damping=0.01)
    assert t.thanos_prune_workspace_bytes(70000, 256, so) == 0
    # the entry point without a workspace argument rejects what its static array cannot hold
    big = t.PruneOpts(mode=t.THANOS_NM, sparsity=0.0, n=2, m=4, block_size=128, damping=0.01)
    assert t.thanos_prune_workspace_bytes(4096, 4096, big) > t.THANOS_NOALLOC_SCRATCH_BYTES
    assert L.thanos_prune_layer_noalloc(fake, t.THANOS_F16, 4096, 4096, fake, ctypes.byref(big),
                                        fake, None, fake, fake, None) == 6


def test_no_oracle_import_in_product():
    # the product path must never route through the CPU oracle
    pkg = os.path.join(ROOT, "paper_2504_05346_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("CPU oracle", ""), f
