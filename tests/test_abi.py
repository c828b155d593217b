"""The C-ABI library loads, exports every symbol include/gear.h declares, and
rejects bad arguments on the host (no GPU needed: nothing is launched)."""
import ctypes
import os
import re

import pytest

from paper_2403_05527_amd import binding as gb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(gb.LIB_PATH):
        from paper_2403_05527_amd.build import build_library
        build_library(verbose=False)
    return gb.load_library()


def test_exports_every_declared_symbol(lib):
    hdr = open(os.path.join(ROOT, "include", "gear.h")).read()
    declared = set(re.findall(r"\b(gear_[a-z_]+)\s*\(", hdr))
    assert declared == set(gb.EXPORTED)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_sizes_match_header():
    assert ctypes.sizeof(gb.gear_config) == 12 * 4
    assert ctypes.sizeof(gb.gear_cache) == 48 + 8 + 8 + 16 + 512


def good():
    return gb.make_config(2, 4, 8, 2, 64, 20000, 20, 512, 4, 4)


def test_cache_bytes_and_invalid_configs(lib):
    a, w = gb.gear_cache_bytes(good())
    assert a > 0 and w > 0 and a % 256 == 0
    bad = [dict(bits=3), dict(group=48), dict(flags=2), dict(d_h=64), dict(H_q=6), dict(H_q=64), dict(n_buf_cap=0),
           dict(n_buf_cap=300), dict(n_prefill_max=0), dict(n_prefill_max=40000), dict(rank_max=9),
           dict(outlier_ppm=-1), dict(n_chunks_max=257), dict(B=0)]
    for kw in bad:
        c = good()
        for k, v in kw.items():
            setattr(c, k, v)
        with pytest.raises(gb.GearError) as e:
            gb.gear_cache_bytes(c)
        assert e.value.status == gb.GEAR_EINVAL, kw


def test_arena_accounting_matches_algorithmic_bytes(lib):
    """Arena size = the algorithmic compressed size (codes + scale/zero + factors +
    4-byte sparse entries, the lists sized for the worst case) + the fixed outlier
    slots (4 per Key token row, 2 per Value channel and 64-token tile, 4 bytes
    each) + the reserved list regions of the Value tiles (48 entries each) + small
    tables and alignment."""
    c = gb.make_config(16, 32, 32, 2, 64, 20000, 20, 4096, 0, 4)
    a, _ = gb.gear_cache_bytes(c)
    slabs, n = 16 * 32, 4096
    algo = 2 * slabs * (n * 128 * 2 // 8 + 4 * (n // 64) * 128 + 2 * n * 4 + 2 * 128 * 4) \
        + 4 * (slabs * 128 * 82 + 16 * n * 82)
    slots = slabs * (n * 4 * 4 + (n // 64) * 128 * 2 * 4 + (n // 64) * 48 * 4)
    assert algo + slots <= a <= (algo + slots) * 1.03


def test_init_and_call_validation_on_host(lib):
    c = good()
    a, w = gb.gear_cache_bytes(c)
    cache = gb.gear_cache()
    fake = ctypes.c_void_p(0x10000000)            # never dereferenced: validation fails first
    assert lib.gear_cache_init(ctypes.byref(c), None, a, ctypes.byref(cache)) == gb.GEAR_EINVAL
    assert lib.gear_cache_init(ctypes.byref(c), ctypes.c_void_p(0x10000010), a, ctypes.byref(cache)) == gb.GEAR_EALIGN
    assert lib.gear_cache_init(ctypes.byref(c), fake, a - 1, ctypes.byref(cache)) == gb.GEAR_ECAPACITY
    assert lib.gear_cache_init(ctypes.byref(c), fake, a, ctypes.byref(cache)) == gb.GEAR_OK
    assert cache.n_total == 0 and cache.n_chunks == 0
    st = None
    # compress: bad n / rank / iters / pointers / capacity -- all rejected before any launch
    assert lib.gear_compress(ctypes.byref(cache), None, fake, 8, 0, 3, None, 0, fake, w, st) == gb.GEAR_EINVAL
    assert lib.gear_compress(ctypes.byref(cache), fake, fake, 0, 0, 3, None, 0, fake, w, st) == gb.GEAR_EINVAL
    assert lib.gear_compress(ctypes.byref(cache), fake, fake, 8, 5, 3, fake, 0, fake, w, st) == gb.GEAR_EINVAL
    assert lib.gear_compress(ctypes.byref(cache), fake, fake, 8, 0, 0, None, 0, fake, w, st) == gb.GEAR_EINVAL
    assert lib.gear_compress(ctypes.byref(cache), fake, fake, 513, 0, 3, None, 0, fake, w, st) == gb.GEAR_ECAPACITY
    assert lib.gear_compress(ctypes.byref(cache), fake, fake, 8, 0, 3, None, 0, fake, w - 1, st) == gb.GEAR_ECAPACITY
    assert lib.gear_compress(ctypes.byref(cache), ctypes.c_void_p(0x10000002), fake, 8, 0, 3, None, 0, fake, w, st) \
        == gb.GEAR_EALIGN
    assert cache.n_total == 0                     # failed calls leave the descriptor untouched
    # decode on an empty cache with an empty buffer is an error; so is n_buf beyond capacity
    assert lib.gear_decode_attn(ctypes.byref(cache), fake, None, None, 0, fake, fake, w, st) == gb.GEAR_EINVAL
    assert lib.gear_decode_attn(ctypes.byref(cache), fake, fake, fake, 21, fake, fake, w, st) == gb.GEAR_EINVAL
    assert lib.gear_decode_attn(ctypes.byref(cache), fake, None, fake, 3, fake, fake, w, st) == gb.GEAR_EINVAL
    assert lib.gear_export_lowrank(ctypes.byref(cache), 0, 0, fake, fake, st) == gb.GEAR_EINVAL
    assert lib.gear_export_codes(ctypes.byref(cache), 2, fake, fake, fake, st) == gb.GEAR_EINVAL
    nnz = ctypes.c_int64(-1)
    assert lib.gear_export_sparse_coo(ctypes.byref(cache), 0, None, None, None, None, 0, st) == gb.GEAR_EINVAL
    assert lib.gear_export_sparse_coo(ctypes.byref(cache), 0, ctypes.byref(nnz), None, None, None, 0, st) == gb.GEAR_OK
    assert nnz.value == 0                         # an empty cache has no outliers
    assert lib.gear_export_sparse_coo(ctypes.byref(cache), 0, ctypes.byref(nnz), fake, None, fake, w, st) == gb.GEAR_EINVAL
    assert gb.strerror(gb.GEAR_ECAPACITY).startswith("capacity")
