"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, rejects bad shapes, and its host-side policy agrees with the
oracle decision for decision (no compute calls that need a GPU)."""
import ctypes as C
import itertools
import os
import re

import numpy as np
import pytest

import paper_2604_19503_amd as R
from paper_2604_19503_amd import binding
from oracle import policy

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = R.load_library()
    header = open(os.path.join(ROOT, "include", "realb.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(realb_[A-Za-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layouts_match_header_field_order():
    header = open(os.path.join(ROOT, "include", "realb.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} realb_config;", header, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = [n for decl in body.split(";") for n in re.findall(r"(\w+)\s*(?:,|$)", decl.strip().split(" ", 1)[-1]) if decl.strip()]
    assert names == [f[0] for f in binding.Config._fields_]


def test_create_rejects_bad_shapes_before_touching_the_gpu():
    lib = R.load_library()
    h = C.c_void_p()
    for kw in (dict(E=64, D=7), dict(k=17), dict(k=65, E=64), dict(H=2000), dict(I=100), dict(E=1024, D=8), dict(E=512, D=4)):
        args = dict(T_max=128, E=64, k=6, D=8, H=2048, I=1408)
        args.update(kw)
        cfg = binding.default_config(**args)
        rc = lib.realb_create(C.byref(cfg), C.byref(h))
        assert rc == -2, (kw, rc)
        assert lib.realb_last_error()
        assert not h.value
    assert lib.realb_create(None, C.byref(h)) == -1


def test_default_config_carries_the_papers_constants():
    cfg = binding.default_config(1, 64, 6, 8, 2048, 1408)
    p = policy.PolicyConfig()
    assert (cfg.C, cfg.tau, cfg.M_init, cfg.aimd_mul, cfg.aimd_add, cfg.Gamma) == (p.C, p.tau, p.M_init, p.aimd_mul, p.aimd_add, p.Gamma)
    assert cfg.aimd_enabled == 1 and cfg.update_first == 1


def test_host_policy_matches_oracle_exhaustively_small():
    n = 0
    for D in (2, 3):
        cfg = binding.default_config(64, 6 * D, 1, D, 128, 128)
        cfg.Gamma = 0
        for total in range(1, 11):
            for load in itertools.product(range(total + 1), repeat=D):
                if sum(load) != total:
                    continue
                for vis in itertools.product(*[sorted({0, l // 2, l}) for l in load]):
                    for M in (0.9, 0.45, 0.0, 1.0):
                        for uf in (1, 0):
                            cfg.update_first = uf
                            want = policy.select_precision(load, vis, total, 1, M, policy.PolicyConfig(Gamma=0, update_first=bool(uf)))
                            got = R.select_precision_host(cfg, load, vis, total, M)
                            assert list(got[0]) == list(want[0]) and got[1] == want[1] and got[2] == want[2], (load, vis, M, uf)
                            n += 1
    assert n > 5000


def test_host_policy_matches_oracle_random_large():
    rng = np.random.default_rng(0)
    for trial in range(400):
        D = int(rng.choice([1, 2, 4, 8, 16]))
        k = int(rng.integers(1, 9))
        T = int(rng.integers(1, 70000))
        w = rng.dirichlet(np.ones(D) * rng.choice([0.3, 1.0, 5.0]))
        load = rng.multinomial(T * k, w)
        vis = (load * rng.uniform(0, 1, D)).astype(np.int64)
        M = float(rng.choice([0.9, 0.45, 0.225, 0.55, 1.0, 0.0, 0.7]))
        aimd = int(rng.integers(0, 2))
        force = int(rng.choice([-1, -1, -1, 0, 1]))
        cfg = binding.default_config(T, 8 * D, k, D, 128, 128)
        cfg.aimd_enabled = aimd
        want = policy.select_precision(load, vis, T, k, M, policy.PolicyConfig(aimd_enabled=bool(aimd)), force)
        got = R.select_precision_host(cfg, load, vis, T, M, force)
        assert list(got[0]) == list(want[0]) and got[1] == want[1] and got[2] == want[2]


def test_host_policy_trajectory_matches_oracle():
    """AIMD state carried over a sequence of layers: fast fall under congestion, slow rise after."""
    cfg = binding.default_config(4096, 64, 6, 8, 2048, 1408)
    M_lib = M_or = 0.9
    rng = np.random.default_rng(1)
    seq = []
    for it in range(40):
        hot = it % 10 < 3
        w = np.ones(8)
        w[it % 8] = 6.0 if hot else 1.2
        load = rng.multinomial(4096 * 6, w / w.sum())
        vis = (load * 0.8).astype(np.int64)
        _, _, M_lib = R.select_precision_host(cfg, load, vis, 4096, M_lib)
        _, _, M_or = policy.select_precision(load, vis, 4096, 6, M_or)
        assert M_lib == M_or
        seq.append(M_lib)
    assert min(seq) < 0.2 and max(seq[5:]) > 0.5


def test_bad_force_value_is_an_error():
    cfg = binding.default_config(64, 8, 2, 1, 128, 128)
    with pytest.raises(R.RealbError):
        R.select_precision_host(cfg, [128], [0], 64, 0.9, force=7)


def test_workspace_bytes_is_host_only_and_matches_its_definition():
    lib = R.load_library()
    cfg = binding.default_config(16384, 64, 6, 8, 2048, 1408)
    n_chunks = -(-16384 * 6 // 256) + 1                                # chunk counts + their sums over groups of 4 chunks
    assert binding.workspace_bytes(cfg) == (n_chunks + -(-n_chunks // 4)) * 8 * 4 + 512 * 2 * 64 * 4
    small = binding.default_config(0, 8, 2, 1, 256, 128)
    assert binding.workspace_bytes(small) == (1 + 1) * 8 * 4 + 512 * 2 * 8 * 4
    bad = binding.default_config(128, 64, 6, 7, 2048, 1408)            # E not a multiple of D
    assert binding.workspace_bytes(bad) == 0 and lib.realb_last_error()
    assert lib.realb_workspace_bytes(None) == 0


def test_scale_offset_and_index_map_describe_the_tiled_layout():
    lib = R.load_library()
    # the layout as the header words it: the 4 scales of one row at one 128-element K-step form a dword,
    # the dwords of 32 consecutive rows are contiguous, K-steps follow, then the next group of 32 rows
    K, rows = 384, 70
    KD = K // 128
    idx = binding.scale_index_map(rows, K)
    assert idx.shape == (rows, K // 32)
    want = np.empty_like(idx)
    pos = 0
    for group in range(-(-rows // 32)):
        for step in range(KD):
            for r in range(32):
                for b in range(4):
                    row = group * 32 + r
                    if row < rows:
                        want[row, step * 4 + b] = pos
                    pos += 1
    assert np.array_equal(idx, want)
    assert len(np.unique(idx)) == idx.size and idx.max() < -(-rows // 32) * 32 * (K // 32)
    for row, kb in ((0, 0), (31, 11), (32, 0), (69, 7)):
        assert lib.realb_scale_offset(row, kb, K) == idx[row, kb]
    bad = C.c_size_t(-1).value
    assert lib.realb_scale_offset(0, 12, K) == bad and lib.realb_scale_offset(-1, 0, K) == bad and lib.realb_scale_offset(0, 0, 100) == bad
    assert lib.realb_scale_index_map(4, 100, None) == -2
    assert lib.realb_scale_index_map(0, 128, None) == 0


def test_gemm_tile_selector_accepts_only_its_values():
    lib = R.load_library()
    for v in (2, 8, 16, 0):
        assert lib.realb_set_gemm_tile(v) == 0
    assert lib.realb_set_gemm_tile(3) == -1
