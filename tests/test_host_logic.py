"""CPU-side checks of the GPU library: it loads, exports the whole C ABI, validates arguments
before touching a device, refuses to run without a GPU, and re-packs meshes losslessly."""
import ctypes
import os
import re

import numpy as np
import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "bps.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bps_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    import paper_2103_07013_amd as bps
    lib = bps.load_library()
    declared = _declared_symbols()
    assert len(declared) >= 10
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in include/bps.h but not exported"
    assert set(declared) == set(bps.EXPORTS)


def test_create_rejects_bad_configs_before_any_device_work():
    import paper_2103_07013_amd as bps
    for kw in (dict(max_batch=0), dict(height=60), dict(width=136), dict(height=4), dict(mode=7),
               dict(threads=320), dict(splits=-1), dict(flags=64), dict(supersample=3), dict(height=72, supersample=2)):
        with pytest.raises(bps.BpsError) as e:
            bps.bps_create(**kw)
        assert e.value.status == -1, kw


def test_no_gpu_means_loud_failure_not_a_fallback():
    import torch
    import paper_2103_07013_amd as bps
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(bps.BpsError) as e:
        bps.bps_create()
    assert e.value.status == -4
    assert "no CPU path" in str(e.value)


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2103_07013_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            assert "paper_2103_07013_amd" not in open(os.path.join(ROOT, "oracle", f)).read()


@pytest.mark.parametrize("which", ["room", "multiroom", "tiny", "soup", "fan", "few_vertices", "loose"])
def test_cluster_packing_is_a_lossless_permutation(which):
    import paper_2103_07013_amd as bps
    if which == "room":
        s = synth.make_room_scene(10_000)
        v, idx = s.vertices, s.indices
    elif which == "multiroom":
        s = synth.make_multiroom_scene(60_000, seed=1002)
        v, idx = s.vertices, s.indices
    elif which == "tiny":
        v = np.array([[0, 0, 0], [1, 0, 0], [0, 1, 0]], np.float32)
        idx = np.array([[0, 1, 2]], np.uint32)
    elif which == "fan":                                             # one hub vertex in 60 000 triangles
        n = 60_000
        ang = np.linspace(0, 2 * np.pi, n + 1)
        v = np.concatenate([[[0, 0, 0]], np.stack([np.cos(ang), np.sin(ang), 0 * ang], 1)]).astype(np.float32)
        idx = np.stack([np.zeros(n, np.int64), np.arange(1, n + 1), np.arange(2, n + 2)], 1).astype(np.uint32)
    elif which == "few_vertices":                                    # every vertex has enormous valence
        rng = np.random.default_rng(3)
        v = rng.uniform(-1, 1, (50, 3)).astype(np.float32)
        idx = rng.integers(0, 50, (60_000, 3)).astype(np.uint32)
    elif which == "loose":                                           # no two triangles share a vertex
        rng = np.random.default_rng(4)
        v = rng.uniform(-5, 5, (90_000, 3)).astype(np.float32)
        idx = np.arange(90_000, dtype=np.uint32).reshape(-1, 3)
    else:
        rng = np.random.default_rng(0)
        v = rng.uniform(-1, 1, (900, 3)).astype(np.float32)
        idx = rng.integers(0, 900, (5000, 3)).astype(np.uint32)      # no locality, repeated indices
    import time
    t0 = time.perf_counter()
    verts, tris, ids = bps.bps_pack_clusters(v, idx)
    assert time.perf_counter() - t0 < 20.0                           # work per cluster is bounded on any mesh
    C = verts.shape[0]
    counts = tris[:, 0] >> 24
    assert counts.min() >= 1 and counts.max() <= 128
    assert counts.sum() == idx.shape[0]
    slot = np.arange(128)[None, :]
    used = slot < counts[:, None]
    assert np.all(ids[~used] == 0xFFFFFFFF)
    assert np.all((tris[~used] & 0xFFFFFF) == 0)
    # every original triangle exactly once
    assert np.array_equal(np.sort(ids[used]), np.arange(idx.shape[0], dtype=np.uint32))
    # local indices lead back to the very same vertex positions
    t = tris & 0xFFFFFF
    cidx = np.repeat(np.arange(C)[:, None], 128, 1)
    for k in range(3):
        li = (t >> (8 * k)) & 0xFF
        assert li[used].max() < 64
        pos = verts[cidx[used], :, li[used]]                         # [n,3]
        assert np.array_equal(pos, v[idx[ids[used], k]])
    if which == "multiroom":
        assert idx.shape[0] / C > 80                                 # patches grown over the mesh are well filled


def test_pack_rejects_out_of_range_index():
    import paper_2103_07013_amd as bps
    v = np.zeros((3, 3), np.float32)
    with pytest.raises(bps.BpsError):
        bps.bps_pack_clusters(v, np.array([[0, 1, 3]], np.uint32))


def test_generators_are_seeded_and_hit_their_triangle_targets():
    a = synth.make_multiroom_scene(50_000, seed=1001)
    b = synth.make_multiroom_scene(50_000, seed=1001)
    c = synth.make_multiroom_scene(50_000, seed=1002)
    assert np.array_equal(a.vertices, b.vertices) and np.array_equal(a.indices, b.indices)
    assert not (a.vertices.shape == c.vertices.shape and np.array_equal(a.vertices, c.vertices))
    assert abs(a.T - 50_000) <= 0.02 * 50_000
    assert a.indices.max() < a.V
    r = synth.make_room_scene(10_000)
    assert abs(r.T - 10_000) <= 0.02 * 10_000
    w1, w2 = synth.build_config(1), synth.build_config(1)
    assert np.array_equal(w1.view_proj, w2.view_proj)
    assert w1.B == 16 and w1.H == 64
