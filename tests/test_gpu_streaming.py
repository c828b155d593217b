"""Decode loop of Algorithm 1 with the streaming buffer: every step pushes the new
token's k/v row into the fp16 buffer, attends over compressed cache + buffer,
and compresses the buffer as a new segment (rank r_g) when it is full.  The HIP
path and the oracle run the same loop on the same bytes; attention is compared
at the first step, around each flush and at the last step."""
import sys

import numpy as np
import pytest
import torch

import gear_workloads as gw
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("bits,n_b,steps", [(2, 20, 45), (4, 7, 30)])
def test_decode_loop_with_flushes(bits, n_b, steps):
    w = gw.Workload("stream", B=2, H_kv=4, H_q=8, n=130, bits=bits, group=64, outlier_ppm=20000, rank=4,
                    rank_chunk=2, n_b=n_b, steps=steps, seed=77 + bits)
    print("case", w, flush=True)
    gc, oc = pu.make_pair(w.B, w.H_kv, w.H_q, w.bits, w.group, w.outlier_ppm, n_b, w.n, steps // n_b + 1, 4)
    K = gw.make_keys(w, w.n, 0, DEV)
    V = gw.make_values(w, w.n, 0, DEV)
    pu.compress_both(gc, oc, K, V, w.rank, w.iters, gw.make_init_B(w, w.rank, 0, DEV))
    Knew = gw.make_keys(w, steps, 5, DEV)          # the tokens the decode steps will produce
    Vnew = gw.make_values(w, steps, 5, DEV)
    Kbuf = torch.zeros(w.B, w.H_kv, n_b, 128, dtype=torch.float16, device=DEV)
    Vbuf = torch.zeros_like(Kbuf)
    n_buf = 0
    flushes = 0
    check = {1, steps}
    for f in range(n_b, steps + 1, n_b):
        check |= {f - 1, f, f + 1}
    for t in range(1, steps + 1):
        Kbuf[:, :, n_buf] = Knew[:, :, t - 1]          # push
        Vbuf[:, :, n_buf] = Vnew[:, :, t - 1]
        n_buf += 1
        if t in check:
            q = gw.make_queries(w, t, DEV)
            rep = pu.compare_attention(gc, oc, q, Kbuf, Vbuf, n_buf)
            print("  step", t, "n_buf", n_buf, "segments", 1 + flushes, rep, flush=True)
        if n_buf == n_b:                                # flush: compress the buffer alone, append
            ib = gw.make_init_B(w, w.rank_chunk, 100 + flushes, DEV)
            pu.compress_both(gc, oc, Kbuf.clone(), Vbuf.clone(), w.rank_chunk, w.iters, ib)
            n_buf = 0
            flushes += 1
    assert gc.n_total == w.n + n_b * (steps // n_b) and n_buf == steps % n_b
    pu.compare_components(gc, oc)
    pu.compare_decompress(gc, oc)
    # a flushed chunk is byte-identical to a fresh compress call on the same tokens
    gc2, _ = pu.make_pair(w.B, w.H_kv, w.H_q, w.bits, w.group, w.outlier_ppm, n_b, n_b, 1, 4)
    Kc = Knew[:, :, :n_b].contiguous()
    Vc = Vnew[:, :, :n_b].contiguous()
    gc2.compress(Kc, Vc, w.rank_chunk, w.iters, gw.make_init_B(w, w.rank_chunk, 100, DEV))
    for which in (0, 1):
        c1, s1, z1 = gc.export_codes(which)
        c2, s2, z2 = gc2.export_codes(which)
        assert torch.equal(c1[:, :, w.n:w.n + n_b], c2)
        m1, v1 = gc.export_sparse(which)
        m2, v2 = gc2.export_sparse(which)
        assert torch.equal(m1[:, :, w.n:w.n + n_b], m2) and torch.equal(v1[:, :, w.n:w.n + n_b], v2)
        A1, B1 = gc.export_lowrank(which, 1)
        A2, B2 = gc2.export_lowrank(which, 0)
        assert torch.equal(A1, A2) and torch.equal(B1, B2)


def test_maximum_chunk_count():
    """A cache filled with the largest number of appended segments the descriptor can hold (GEAR_MAX_CHUNKS), of
    mixed lengths and ranks: components, reconstruction and attention against the oracle; one more compress call is
    refused on the host."""
    nmax = pu.gb.GEAR_MAX_CHUNKS
    w = gw.Workload("maxchunks", B=1, H_kv=2, H_q=4, n=70, bits=2, group=64, outlier_ppm=20000, rank=2,
                    rank_chunk=2, n_b=8, steps=1, seed=321)
    print("case", w, flush=True)
    gc, oc = pu.make_pair(w.B, w.H_kv, w.H_q, w.bits, w.group, w.outlier_ppm, w.n_b, w.n, nmax, 2)
    pu.compress_both(gc, oc, gw.make_keys(w, w.n, 0, DEV), gw.make_values(w, w.n, 0, DEV), 2, 3, gw.make_init_B(w, 2, 0, DEV))
    for j in range(nmax):
        nj, rj = 1 + j % w.n_b, j % 3
        pu.compress_both(gc, oc, gw.make_keys(w, nj, 1 + j, DEV), gw.make_values(w, nj, 1 + j, DEV), rj, 3,
                         gw.make_init_B(w, rj, 1 + j, DEV))
    with pytest.raises(pu.gb.GearError) as e:
        gc.compress(gw.make_keys(w, 1, 999, DEV), gw.make_values(w, 1, 999, DEV), 0, 3)
    assert e.value.status == pu.gb.GEAR_ECAPACITY
    rep = pu.compare_components(gc, oc)
    rep.update(pu.compare_decompress(gc, oc))
    Kb, Vb = gw.make_keys(w, w.n_b, 50, DEV), gw.make_values(w, w.n_b, 50, DEV)
    rep.update(pu.compare_attention(gc, oc, gw.make_queries(w, 0, DEV), Kb, Vb, 5))
    print("  ->", rep, flush=True)


def test_maximum_buffer_capacity():
    """n_b = 255, the largest streaming buffer: 255 live fp16 rows in the decode read, and flushed segments of 255
    and 129 tokens (two 128-row pieces per chunk in the decode kernel) next to a short one."""
    w = gw.Workload("maxbuf", B=2, H_kv=2, H_q=4, n=300, bits=4, group=32, outlier_ppm=20000, rank=4,
                    rank_chunk=2, n_b=255, steps=1, seed=654)
    print("case", w, flush=True)
    gc, oc = pu.make_pair(w.B, w.H_kv, w.H_q, w.bits, w.group, w.outlier_ppm, 255, w.n, 3, 4)
    pu.compress_both(gc, oc, gw.make_keys(w, w.n, 0, DEV), gw.make_values(w, w.n, 0, DEV), 4, 3, gw.make_init_B(w, 4, 0, DEV))
    for j, nj in enumerate((255, 129, 20)):
        pu.compress_both(gc, oc, gw.make_keys(w, nj, 1 + j, DEV), gw.make_values(w, nj, 1 + j, DEV), 2, 3,
                         gw.make_init_B(w, 2, 1 + j, DEV))
    rep = pu.compare_components(gc, oc)
    rep.update(pu.compare_decompress(gc, oc))
    Kb, Vb = gw.make_keys(w, 255, 50, DEV), gw.make_values(w, 255, 50, DEV)
    q = gw.make_queries(w, 0, DEV)
    for n_buf in (255, 128, 1):
        r = pu.compare_attention(gc, oc, q, Kb, Vb, n_buf)
        rep["attn_bar_used_%d" % n_buf] = r["attn_bar_used"]
    print("  ->", rep, flush=True)
