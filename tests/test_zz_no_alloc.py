"""gear_decode_attn_static (the entry point for callers that cannot allocate: its split
records live in a fixed array inside the library) against gear_decode_attn, through the
C ABI, on two calls in a row, the second on a smaller cache: the same kernels write the
same records, so the outputs must agree bit for bit; the first is also held to the
attention bar against the oracle.  A cache whose records exceed the array is refused."""
import ctypes

import pytest
import torch

import gear_workloads as gw
from paper_2403_05527_amd import binding as gb
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def build_cache(w, n_chunks, with_oracle):
    gc, oc = pu.make_pair(w.B, w.H_kv, w.H_q, w.bits, w.group, w.outlier_ppm, w.n_b, w.n, max(n_chunks, 1),
                          max(w.rank, w.rank_chunk))
    K, V = gw.make_keys(w, w.n, 0, DEV), gw.make_values(w, w.n, 0, DEV)
    ib = gw.make_init_B(w, w.rank, 0, DEV)
    if with_oracle:
        pu.compress_both(gc, oc, K, V, w.rank, w.iters, ib)
    else:
        gc.compress(K, V, w.rank, w.iters, ib)
    for j in range(n_chunks):
        Kc, Vc = gw.make_keys(w, w.n_b, 1 + j, DEV), gw.make_values(w, w.n_b, 1 + j, DEV)
        ibc = gw.make_init_B(w, w.rank_chunk, 1 + j, DEV)
        if with_oracle:
            pu.compress_both(gc, oc, Kc, Vc, w.rank_chunk, w.iters, ibc)
        else:
            gc.compress(Kc, Vc, w.rank_chunk, w.iters, ibc)
    return gc, oc


def both_entry_points(gc, w, n_buf, stream_q):
    q = gw.make_queries(w, stream_q, DEV)
    Kb, Vb = gw.make_keys(w, w.n_b, 50, DEV), gw.make_values(w, w.n_b, 50, DEV)
    ref = torch.empty_like(q)
    gb.gear_decode_attn(gc.cache, q, Kb, Vb, n_buf, ref, gc.workspace)
    out = torch.full_like(q, float("nan"))
    gb.gear_decode_attn_static(gc.cache, q, Kb, Vb, n_buf, out)
    torch.cuda.synchronize()
    return q, Kb, Vb, ref, out


def test_static_scratch_entry_point_matches_workspace_entry_point():
    big = gw.Workload("static_a", B=2, H_kv=4, H_q=8, n=1300, bits=2, group=64, outlier_ppm=20000, rank=4,
                      rank_chunk=2, n_b=20, steps=1, seed=61)
    print("case", big, flush=True)
    gc, oc = build_cache(big, 5, True)
    q, Kb, Vb, ref, out = both_entry_points(gc, big, 7, 0)
    assert torch.equal(out, ref)
    oc.decode_attn(pu.np16(q), pu.np16(Kb), pu.np16(Vb), 7)
    print("  first call", pu.check_attention(pu.np16(out), oc.last_attn_f64), flush=True)
    # second call right after, on a smaller cache (fewer records: the array still holds the first call's)
    small = gw.Workload("static_b", B=1, H_kv=2, H_q=2, n=90, bits=4, group=32, outlier_ppm=10000, rank=2,
                        rank_chunk=2, n_b=20, steps=1, seed=62)
    print("case", small, flush=True)
    gc2, oc2 = build_cache(small, 1, True)
    q, Kb, Vb, ref, out = both_entry_points(gc2, small, 20, 1)
    assert torch.equal(out, ref)
    oc2.decode_attn(pu.np16(q), pu.np16(Kb), pu.np16(Vb), 20)
    print("  second call", pu.check_attention(pu.np16(out), oc2.last_attn_f64), flush=True)
    # and the first cache once more: nothing of the second call is left in its way
    q, Kb, Vb, ref, out = both_entry_points(gc, big, 3, 2)
    assert torch.equal(out, ref)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    # records of this cache: 64 * 64 * (64 + 1) * 520 bytes = 138 MB > 32 MiB; nothing is launched
    cfg = gb.make_config(64, 8, 64, 2, 64, 0, 20, 32768, 1, 0)
    a, _ = gb.gear_cache_bytes(cfg)
    cache = gb.gear_cache()
    fake = ctypes.c_void_p(0x10000000)                       # never dereferenced
    lib = gb.load_library()
    assert lib.gear_cache_init(ctypes.byref(cfg), fake, a, ctypes.byref(cache)) == gb.GEAR_OK
    cache.n_prefill = cache.n_total = 32768
    assert lib.gear_decode_attn_static(ctypes.byref(cache), fake, None, None, 0, fake, None) == gb.GEAR_ECAPACITY
    assert lib.gear_decode_attn_static(ctypes.byref(cache), None, None, None, 0, fake, None) == gb.GEAR_EINVAL
