"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, builds the level table of Eq. 2-3 exactly as the oracle does
(the two are written independently) and reports errors as status codes."""
import ctypes
import os
import re

import pytest

from oracle import hashgrid_oracle as orc
from paper_2201_05989_amd import binding
from paper_2201_05989_amd.build import LIB_PATH, PROBES_LIB_PATH

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hashgrid_[a-z_]+)\s*\(", text)))


def test_library_is_built_and_exports_every_declared_symbol():
    assert os.path.exists(LIB_PATH), "build the library first: __graft_entry__.build()"
    lib = ctypes.CDLL(LIB_PATH)
    names = _declared_symbols("hashgrid.h")
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n
    assert not any("probe" in n for n in names)  # measurement tooling is not behind the method's ABI


def test_probe_library_is_built_and_exports_every_declared_symbol():
    assert os.path.exists(PROBES_LIB_PATH), "build the probes first: __graft_entry__.build()"
    lib = ctypes.CDLL(PROBES_LIB_PATH)
    names = _declared_symbols("hashgrid_probes.h")
    assert set(names) == set(binding.PROBE_EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


CFGS = [(2, 4, 2, 1 << 10, 4, 32), (2, 16, 2, 1 << 22, 16, 32768), (3, 16, 2, 1 << 19, 16, 2048),
        (3, 16, 2, 1 << 24, 16, 524288), (3, 16, 2, 1 << 19, 16, 512), (3, 16, 2, 1 << 14, 16, 4096),
        (2, 16, 2, 1 << 22, 16, 11733), (3, 8, 4, 1 << 19, 16, 1000), (3, 32, 1, 1 << 19, 16, 2048),
        (1, 7, 8, 100, 3, 999), (3, 1, 2, 1 << 12, 16, 16), (3, 16, 2, 1000003, 16, 2048),
        (2, 16, 2, 1 << 17, 16, 11733), (3, 16, 2, 1 << 21, 16, 8192), (3, 12, 2, 1 << 15, 5, 77)]


@pytest.mark.parametrize("interp", [0, 1])
@pytest.mark.parametrize("d,L,F,T,N_min,N_max", CFGS)
def test_level_table_matches_oracle(d, L, F, T, N_min, N_max, interp):
    g = binding.HashGrid(d, L, F, T, N_min, N_max, "f16", "f16", interp)
    lv = orc.levels(orc.OracleConfig(d, L, F, T, N_min, N_max, interp))
    assert g.n_entries == lv.total
    for l, info in enumerate(g.levels()):
        assert (info.N, info.entry_offset, info.n_entries, info.is_dense) == \
            (int(lv.N[l]), int(lv.offset[l]), int(lv.size[l]), bool(lv.dense[l]))


def test_level_table_sweep_of_resolutions_matches_oracle():
    # every N_max in a range, three level counts: the two floor() evaluations must never disagree
    for L in (2, 9, 16):
        for N_max in list(range(16, 700)) + [2 ** k for k in range(10, 20)]:
            g = binding.HashGrid(3, L, 2, 1 << 16, 16, N_max)
            lv = orc.levels(orc.OracleConfig(3, L, 2, 1 << 16, 16, N_max))
            assert [i.N for i in g.levels()] == list(map(int, lv.N)), (L, N_max)


def _create(**kw):
    base = dict(d=3, L=16, F=2, T=1 << 19, N_min=16, N_max=2048, param_dtype=1, io_dtype=1, interp=0, grad_dtype=0)
    base.update(kw)
    lib = binding.load_library()
    cfg = binding.hashgrid_config(*[base[k] for k, _ in binding.hashgrid_config._fields_])
    h = ctypes.c_void_p()
    st = lib.hashgrid_create(ctypes.byref(cfg), ctypes.byref(h))
    if st == 0:
        lib.hashgrid_destroy(h)
    return st


def test_create_status_codes():
    assert _create() == 0 and _create(grad_dtype=1) == 0
    for bad in (dict(d=0), dict(L=0), dict(F=0), dict(T=0), dict(N_min=0), dict(N_max=8), dict(param_dtype=2),
                dict(io_dtype=7), dict(interp=2), dict(grad_dtype=2)):
        assert _create(**bad) == 1, bad  # HG_ERR_INVALID_ARG
    for unsup in (dict(d=4), dict(L=33), dict(F=3), dict(F=16)):
        assert _create(**unsup) == 2, unsup  # HG_ERR_UNSUPPORTED
    lib = binding.load_library()
    assert lib.hashgrid_create(None, None) == 1
    assert lib.hashgrid_n_entries(None) == 0
    lib.hashgrid_destroy(None)
    assert binding.strerror(0) == "ok" and "unsupported" in binding.strerror(2)


def test_null_and_empty_batches_need_no_device():
    lib = binding.load_library()
    g = binding.HashGrid(2, 4, 2, 1 << 10, 4, 32, "f32", "f32")
    assert lib.hashgrid_encode_fwd(g._h, 0, None, None, None, None) == 0   # B = 0: nothing to do
    assert lib.hashgrid_encode_bwd(g._h, 0, None, None, None, None) == 0
    assert lib.hashgrid_encode_fwd(g._h, 8, None, None, None, None) == 1   # NULL data pointers
    assert lib.hashgrid_encode_bwd(g._h, 8, None, None, None, None) == 1
    assert lib.hashgrid_encode_bwd_input(g._h, 8, None, None, None, None, None) == 1
    assert lib.hashgrid_encode_fwd(None, 8, None, None, None, None) == 1
    assert lib.hashgrid_level_info(g._h, 4, None, None, None, None) == 1   # level out of range
    assert lib.hashgrid_level_info(g._h, 3, None, None, None, None) == 0
    assert lib.hashgrid_debug_indices(g._h, 8, None, 9, None, None, None) == 1
    assert lib.hashgrid_debug_count_outside(g._h, 8, 4096, None, None) == 1   # no counter
    assert lib.hashgrid_debug_count_outside(g._h, 8, None, 4096, None) == 1   # no points
    assert lib.hashgrid_debug_count_outside(g._h, 0, None, 4096, None) == 0   # B = 0
    # more than HG_MAX_BATCH (2^28) points per call: refused before anything is launched
    big = (1 << 28) + 1
    assert lib.hashgrid_encode_fwd(g._h, big, 4096, 4096, 4096, None) == 2
    assert lib.hashgrid_encode_bwd(g._h, big, 4096, 4096, 4096, None) == 2
    assert lib.hashgrid_encode_bwd_input(g._h, big, 4096, 4096, 4096, 4096, None) == 2
    assert lib.hashgrid_debug_indices(g._h, big, 4096, 0, 4096, 4096, None) == 2
    assert lib.hashgrid_bwd_workspace_bytes(g._h, big) == 0
    # misaligned pointers are rejected before any launch (F*sizeof = 8-byte vectors here)
    assert lib.hashgrid_encode_fwd(g._h, 8, 4096, 4100, 4096, None) == 1


def test_adam_step_status_codes_need_no_device():
    lib = binding.load_library()
    cfg = binding.hashgrid_adam_config(1e-2, 0.9, 0.99, 1e-15, 0.0)
    assert lib.hashgrid_adam_step(0, None, None, None, None, None, ctypes.byref(cfg), 1, 1, None) == 0
    assert lib.hashgrid_adam_step(8, None, None, None, None, None, ctypes.byref(cfg), 1, 1, None) == 1
    assert lib.hashgrid_adam_step(8, 4096, None, 4096, 4096, 4096, ctypes.byref(cfg), 0, 1, None) == 1
    assert lib.hashgrid_adam_step(8, 4096, None, 4096, 4096, 4096, None, 1, 1, None) == 1


def test_probe_status_codes_need_no_device():
    lib = binding.load_probes()
    assert lib.hashgrid_probe_copy(None, None, 0, None) == 0
    assert lib.hashgrid_probe_copy(None, 4096, 64, None) == 1
    assert lib.hashgrid_probe_copy(4096, 8192, 24, None) == 1      # not a multiple of 16
    assert lib.hashgrid_probe_copy(4100, 8192, 64, None) == 1      # misaligned
    assert lib.hashgrid_probe_gather(None, 1024, 0, 1, None, None) == 0
    assert lib.hashgrid_probe_gather(4096, 1000, 4096, 1, 8192, None) == 1   # table not a power of two
    assert lib.hashgrid_probe_gather(4096, 1024, 100, 1, 8192, None) == 1    # not a multiple of 4096
    assert lib.hashgrid_probe_atomic_add(None, 1024, 4096, 1, None) == 1
    assert lib.hashgrid_probe_atomic_add(4096, 1 << 33, 4096, 1, None) == 1
    assert lib.hashgrid_probe_gather_lines(None, 1024, 1, 0, 16, 1, None, None) == 0
    assert lib.hashgrid_probe_gather_lines(4096, 1000, 1, 1024, 16, 1, 8192, None) == 1   # slice not a power of two
    assert lib.hashgrid_probe_gather_lines(4096, 1024, 1, 1000, 16, 1, 8192, None) == 1   # not a multiple of 1024
    assert lib.hashgrid_probe_gather_lines(4096, 1024, 0, 1024, 16, 1, 8192, None) == 1   # no slice


def test_encode_mlp_status_codes_need_no_device():
    g = binding.HashGrid(3, 16, 2, 1 << 19, 16, 2048, "f32", "f16")   # fp32 tables
    lib = g._lib
    assert lib.hashgrid_encode_mlp_fwd(g._h, 8, 4096, 4096, 4096, 4096, 4096, 1, 4096, None) == 2
    g = binding.HashGrid(3, 16, 8, 1 << 19, 16, 2048)                 # 128 inputs
    assert lib.hashgrid_encode_mlp_fwd(g._h, 8, 4096, 4096, 4096, 4096, 4096, 1, 4096, None) == 2
    g = binding.HashGrid(3, 16, 2, 1 << 19, 16, 2048)
    assert lib.hashgrid_encode_mlp_fwd(g._h, 8, 4096, 4096, 4096, 4096, 4096, 33, 4096, None) == 2
    assert lib.hashgrid_encode_mlp_fwd(g._h, 8, 4096, 4096, 4096, 4096, 4096, 0, 4096, None) == 1
    assert lib.hashgrid_encode_mlp_fwd(g._h, 8, None, 4096, 4096, 4096, 4096, 1, 4096, None) == 1
    assert lib.hashgrid_encode_mlp_fwd(g._h, 0, None, None, None, None, None, 1, None, None) == 0


def test_choice_between_the_backward_passes_needs_no_device():
    """hashgrid_bwd_ws_pays is host arithmetic on sizes: the sort for large batches, atomics for small
    ones, and the sort again where a small batch would queue its atomics on a handful of entries."""
    table1 = binding.HashGrid(3, 16, 2, 1 << 19, 16, 2048)
    assert not table1.bwd_ws_pays(1024) and not table1.bwd_ws_pays(4096)
    assert table1.bwd_ws_pays(1 << 14) and table1.bwd_ws_pays(1 << 18)
    small_levels = binding.HashGrid(2, 4, 2, 1 << 10, 4, 32, "f32", "f32")  # level 0 has 25 entries
    assert not small_levels.bwd_ws_pays(512) and small_levels.bwd_ws_pays(4096)
    odd = binding.HashGrid(3, 16, 2, 1000003, 16, 2048)  # T not 2^k: a record per corner, twice as many
    assert odd.bwd_ws_pays(1 << 20) and not odd.bwd_ws_pays(4096)
    assert not binding.HashGrid(3, 2, 2, 1 << 25, 16, 2048).bwd_ws_pays(1 << 20)  # not served: too many chunks
    wide = binding.HashGrid(3, 16, 8, 1 << 19, 16, 2048, "f16", "f32")  # 40-byte records: pays later
    first = [min(k for k in range(6, 22) if g.bwd_ws_pays(1 << k)) for g in (table1, wide)]
    assert first[0] <= first[1]
    for grid in (table1, small_levels, odd, wide):  # once it pays it keeps paying
        flags = [grid.bwd_ws_pays(1 << k) for k in range(6, 22)]
        assert flags == sorted(flags)


def test_workspace_size_of_the_sorted_backward_needs_no_device():
    """hashgrid_bwd_workspace_bytes is host arithmetic: 8 + F * sizeof(dL/dy scalar) bytes per pair of
    corners plus one count per (tile, chunk); 0 where the pass is not served."""
    B = 1 << 18
    table1 = binding.HashGrid(3, 16, 2, 1 << 19, 16, 2048, "f16", "f16")
    pairs = B * 16 * 4
    chunks = sum(-(-lv.n_entries // 4096) if not lv.is_dense else 0 for lv in table1.levels())
    assert chunks == 11 * 128
    need = table1.bwd_workspace_bytes(B)
    assert pairs * 12 + (B // 512) * chunks * 4 < need < pairs * 12 + (B // 512 + 2) * (chunks + 200) * 4 + (1 << 16)
    assert binding.HashGrid(3, 16, 2, 1 << 19, 16, 2048, "f16", "f32").bwd_workspace_bytes(B) - need == pairs * 4
    assert binding.HashGrid(3, 16, 8, 1 << 19, 16, 2048, "f16", "f16").bwd_workspace_bytes(B) > pairs * 24
    # more than 16384 chunks: tiles of 4096 points, an eighth of the count rows
    large = binding.HashGrid(3, 16, 2, 1 << 24, 16, 1 << 19, "f16", "f16")
    need = large.bwd_workspace_bytes(1 << 21)
    assert (1 << 21) * 16 * 4 * 12 < need < (1 << 21) * 16 * 4 * 12 + 600 * 50000 * 4
    # not served: one dimension, T not a power of two, T beyond 2^24, too many pairs for 32-bit slots
    # one record per corner where the pairing along dimension 0 does not hold: d = 1, T not a power of two
    assert binding.HashGrid(1, 4, 2, 1 << 10, 4, 64).bwd_workspace_bytes(1000) > 1000 * 4 * 2 * 12
    odd = binding.HashGrid(3, 16, 2, 1000003, 16, 2048).bwd_workspace_bytes(1000)
    assert 1000 * 16 * 8 * 12 < odd < 1000 * 16 * 8 * 12 + (1 << 20)
    assert binding.HashGrid(3, 2, 2, 1 << 25, 16, 2048).bwd_workspace_bytes(1000) == 0
    assert table1.bwd_workspace_bytes(1 << 27) == 0
    assert table1.bwd_workspace_bytes(0) == 0
