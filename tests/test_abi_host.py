"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and rejects
bad arguments with error codes before touching the GPU."""
import ctypes
import os
import re

import pytest

import paper_2512_20920_amd as R

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(R.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return R.load_library()


def good_cfg(**kw):
    base = dict(d_model=64, n_heads=4, head_dim=16, n_experts=8, top_k=2, d_expert=128, d_shared=0, dtype=0,
                causal=1, use_rope=1, norm_topk_prob=0, n_inv_iters=1, rope_theta=1e6, rms_eps=1e-6)
    base.update(kw)
    return R.Config(**base)


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "revffn.h")).read()
    declared = set(re.findall(r"\b(revffn_[a-z_]+)\s*\(", header))
    assert declared == set(R.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def header_text():
    return open(os.path.join(ROOT, "include", "revffn.h")).read()


def test_struct_layouts_match_header():
    assert ctypes.sizeof(R.Config) == 17 * 4
    cbody = header_text()[header_text().index("typedef struct revffn_config {"):header_text().index("} revffn_config;")]
    assert tuple(re.findall(r"(?:int32_t|float)\s+([a-z_0-9]+);", cbody)) == tuple(n for n, _ in R.Config._fields_)
    assert ctypes.sizeof(R.Weights) == 21 * ctypes.sizeof(ctypes.c_void_p)
    assert ctypes.sizeof(R.Grads) == ctypes.sizeof(R.Weights)
    header = open(os.path.join(ROOT, "include", "revffn.h")).read()
    body = header[header.index("typedef struct revffn_weights {"):header.index("} revffn_weights;")]
    order = re.findall(r"\*\s*([a-z_0-9]+)\s*[,;]", body)
    assert tuple(order) == R.WEIGHT_FIELDS


def test_workspace_bytes_and_bad_configs(lib):
    cfg = good_cfg()
    n = lib.revffn_workspace_bytes(ctypes.byref(cfg), 2, 32)
    assert n > 0
    assert lib.revffn_workspace_bytes(ctypes.byref(cfg), 4, 32) > n
    bad = [dict(d_model=63), dict(n_heads=3), dict(top_k=0), dict(top_k=9), dict(n_experts=0), dict(dtype=2),
           dict(head_dim=15, n_heads=4, d_model=60), dict(n_inv_iters=-1), dict(rope_theta=0.0), dict(d_expert=0),
           dict(n_experts=300, top_k=2), dict(top_k=17, n_experts=32), dict(fp32_streams=2), dict(symmetric=-1), dict(fp32_grads=3)]
    for kw in bad:
        c = good_cfg(**kw)
        assert lib.revffn_workspace_bytes(ctypes.byref(c), 2, 32) == 0, kw
        h = ctypes.c_void_p()
        assert lib.revffn_create(ctypes.byref(h), ctypes.byref(c), 2, 32) == -1, kw
        assert not h.value
    h = ctypes.c_void_p()
    assert lib.revffn_create(ctypes.byref(h), ctypes.byref(cfg), 0, 32) == -2
    assert lib.revffn_create(None, ctypes.byref(cfg), 2, 32) == -3
    assert lib.revffn_create(ctypes.byref(h), None, 2, 32) == -3


def test_null_context_and_strerror(lib):
    w = R.Weights()
    assert lib.revffn_forward(None, ctypes.byref(w), 1, 1, 1, 1, 1, 1, 32, None) == -3
    assert lib.revffn_inverse(None, ctypes.byref(w), 1, 1, 1, 1, 1, 1, 32, None, None) == -3
    assert lib.revffn_backward(None, ctypes.byref(w), 1, 1, 1, 1, 1, 1, 1, None, 1, 1, 32, None) == -3
    m = R.Merged()
    assert lib.revffn_merge_adapters(None, ctypes.byref(w), ctypes.byref(m), None) == -3
    assert lib.revffn_forward_merged(None, ctypes.byref(w), ctypes.byref(m), 1, 1, 1, 1, 1, 1, 32, None) == -3
    assert lib.revffn_inverse_merged(None, ctypes.byref(w), ctypes.byref(m), 1, 1, 1, 1, 1, 1, 32, None, None) == -3
    assert lib.revffn_get_routing(None, None, None, None, None, None, None) == -3
    assert lib.revffn_set_inv_iters(None, 1) == -3
    assert lib.revffn_set_inverse_tolerance(None, 1e-3, 4) == -3
    assert lib.revffn_get_inverse_stats(None, None, None, None, None) == -3
    lib.revffn_destroy(None)
    seen = set()
    for code in range(0, -7, -1):
        msg = R.revffn_strerror(code)
        assert msg and msg != "unknown error"
        seen.add(msg)
    assert len(seen) == 7 and R.revffn_strerror(-99) == "unknown error"


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2512_20920_amd.binding as bnd
    monkeypatch.setattr(bnd, "_LIB", None)
    monkeypatch.setattr(bnd, "_HERE", str(tmp_path))
    with pytest.raises(R.RevffnError):
        bnd.load_library()


def test_tile_placement_covers_every_tile_once():
    """The XCD-aware workgroup -> tile map of the MFMA GEMM (the same index function the kernel runs, evaluated on
    the host by the library) is a bijection onto the tiles: no tile twice, none missing, no tile out of range."""
    import numpy as np
    R = pytest.importorskip("paper_2512_20920_amd")
    rng = np.random.default_rng(0)
    # dense problems, including tile grids that the 2-D split over 8 XCDs does not divide evenly
    for tiles_m, tiles_n in [(8, 8), (16, 32), (9, 21), (17, 5), (1, 64), (64, 1), (3, 88), (33, 7), (16, 176)]:
        for bm, bn in [(128, 128), (128, 64)]:
            wg = R.revffn_op_tile_placement(0, tiles_m, tiles_n, bm, bn)
            live = wg[wg[:, 0] >= 0]
            assert len(live) == tiles_m * tiles_n and len(wg) % 8 == 0
            assert live[:, 0].max() < tiles_n and live[:, 1].max() < tiles_m
            assert len({(int(x), int(y)) for x, y, _ in live}) == tiles_m * tiles_n
    # expert tile lists: random tiles per expert (some experts empty), unused slots after the last tile
    for _ in range(40):
        tiles_n = int(rng.integers(1, 30))
        per_expert = rng.integers(0, 5, size=int(rng.integers(1, 24)))
        first = np.concatenate([[0], np.cumsum(per_expert)])
        tf = np.concatenate([np.full(c, (f << 16) | c, dtype=np.int32) for f, c in zip(first[:-1], per_expert)]
                            + [np.zeros(0, np.int32)])
        n_used = int(per_expert.sum())
        for use_first in (True, False):
            wg = R.revffn_op_tile_placement(1, n_used + 7, tiles_n, 128, 128, 1, tf if use_first else None, n_used)
            live = wg[wg[:, 0] >= 0]
            assert len(live) == tiles_n * n_used
            if n_used:
                assert live[:, 0].max() < tiles_n and live[:, 1].max() < n_used
            assert len({(int(x), int(y)) for x, y, _ in live}) == tiles_n * n_used
            if use_first and n_used:
                # the m-tiles of one expert and one n-tile are consecutive workgroups of one XCD
                order = {(int(x), int(y)): i for i, (x, y, _) in enumerate(wg) if x >= 0}
                for f, c in zip(first[:-1], per_expert):
                    for j in range(1, int(c)):
                        a, b = order[(0, int(f) + j - 1)], order[(0, int(f) + j)]
                        assert (a & 7) != (b & 7) or b - a == 8
    # per-expert weight gradients: every (expert, tile) once, under both placements and for tile counts and expert
    # counts that the split over XCD pairs does not divide evenly; with an even routing an expert stays on two XCDs
    for tiles_m, tiles_n, E in [(3, 5, 13), (11, 8, 60), (8, 6, 60), (1, 1, 1), (2, 9, 7)]:
        for even in (1, 0):
            wg = R.revffn_op_tile_placement(2, tiles_m, tiles_n, 256, 256, n_groups=E, n_used=even)
            live = wg[wg[:, 0] >= 0]
            assert len(live) == E * tiles_m * tiles_n and len({tuple(map(int, r)) for r in live}) == E * tiles_m * tiles_n
            assert live[:, 0].max() < tiles_n and live[:, 1].max() < tiles_m and live[:, 2].max() < E
            if even:
                xcd = np.arange(len(wg)) & 7
                for e in range(E):
                    used = set(xcd[(wg[:, 2] == e)])
                    assert len(used) <= 2 and len({x >> 1 for x in used}) == 1
