"""GPU parity at the benchmark's full sizes (configs 1-4 and the GEAR-L variant
of config 4), in the launch configuration bench.py times.  The whole batch runs
on the GPU; the oracle recomputes one sampled batch element (a subset of heads
for the long-context config) from the same bytes, which is exact: Keys are
independent per (batch, head), Values per batch element (their Filter ranks a
token across all heads, so the support of S is computed on all heads even when
only some heads are then compared).  Bars are those of test_gpu_parity.py."""
import sys

import numpy as np
import pytest
import torch

import gear_workloads as gw
from oracle import gear_oracle as go
from paper_2403_05527_amd import binding as gb
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def host(t):
    return t.detach().cpu().numpy()


def run_full(w, b_sel, heads, n_buf):
    say("full-size case", w.name, "sampled batch element", b_sel, "heads", heads)
    H = w.H_kv
    heads = list(range(H)) if heads is None else heads
    gq = w.H_q // H
    qheads = [h * gq + i for h in heads for i in range(gq)]
    cfg = gb.make_config(w.B, H, w.H_q, w.bits, w.group, w.outlier_ppm, w.n_b, w.n, 2, max(w.rank, w.rank_chunk))
    gc = gb.GearCache(cfg, DEV)
    oc = go.OracleCache(1, len(heads), len(qheads), 128, w.bits, w.group, w.outlier_ppm)

    def both(K, V, rank, ib):
        gc.compress(K, V, rank, w.iters, ib)
        Kb, Vb = host(K[b_sel:b_sel + 1]), host(V[b_sel:b_sel + 1])
        v_mask = go.filter_values(Vb, w.outlier_ppm)[:, heads] if w.outlier_ppm > 0 else None
        oc.compress(np.ascontiguousarray(Kb[:, heads]), np.ascontiguousarray(Vb[:, heads]), rank, w.iters,
                    np.ascontiguousarray(host(ib[:, b_sel:b_sel + 1])[:, :, heads]), v_mask)

    K = gw.make_keys(w, w.n, 0, DEV)
    V = gw.make_values(w, w.n, 0, DEV)
    both(K, V, w.rank, gw.make_init_B(w, w.rank, 0, DEV))
    del K, V
    Kc = gw.make_keys(w, w.n_b, 1, DEV)
    Vc = gw.make_values(w, w.n_b, 1, DEV)
    both(Kc, Vc, w.rank_chunk, gw.make_init_B(w, w.rank_chunk, 1, DEV))

    rep = {}
    sl = lambda t: host(t[b_sel:b_sel + 1])[:, heads]
    for which, (name, segs) in enumerate((("K", oc.K), ("V", oc.V))):
        codes, scale, zero = [sl(x) for x in gc.export_codes(which)]
        o_codes = np.concatenate([s.codes for s in segs], axis=2)
        assert np.array_equal(scale.astype(np.float32),
                              np.concatenate([s.scale for s in segs], axis=2).astype(np.float32)), name + " scale"
        assert np.array_equal(zero.astype(np.float32),
                              np.concatenate([s.zero for s in segs], axis=2).astype(np.float32)), name + " zero"
        mism = int(np.count_nonzero(codes != o_codes))
        ties = sum(s.ties for s in segs)
        rep[name + "_code_mismatches"], rep[name + "_exact_ties"] = mism, ties
        assert mism == 0 or (mism <= ties and np.abs(codes.astype(int) - o_codes.astype(int)).max() <= 1), name
        del codes, scale, zero
        mask, vals = [sl(x) for x in gc.export_sparse(which)]
        o_mask = np.concatenate([s.mask for s in segs], axis=2)
        o_vals = np.concatenate([s.svals for s in segs], axis=2)
        assert np.array_equal(mask.astype(bool), o_mask), name + " outlier support"
        assert np.array_equal(vals.view(np.uint16), o_vals.view(np.uint16)), name + " outlier values"
        rep[name + "_nnz"] = int(o_mask.sum())
        del mask, vals
    Kg, Vg = gc.decompress()
    Ko, Vo = oc.decompress()
    rep["K_rel_frob"], rep["V_rel_frob"] = pu.rel_frob(sl(Kg), Ko), pu.rel_frob(sl(Vg), Vo)
    assert rep["K_rel_frob"] <= pu.REL_FROB_TOL and rep["V_rel_frob"] <= pu.REL_FROB_TOL, rep
    del Kg, Vg
    # invariants that hold at any size, checked on the whole batch: exact outlier counts per vector
    if w.outlier_ppm > 0:
        mk, _ = gc.export_sparse(0)
        kv_n = go.outlier_counts(w.n, w.outlier_ppm)[0]
        kv_c = go.outlier_counts(w.n_b, w.outlier_ppm)[0]
        assert (mk[:, :, :w.n].sum(dim=2) == kv_n).all() and (mk[:, :, w.n:].sum(dim=2) == kv_c).all()
        del mk
        mv, _ = gc.export_sparse(1)
        assert (mv.sum(dim=(1, 3)) == go.outlier_counts(H * 128, w.outlier_ppm)[0]).all()
        del mv
    # decode attention over prefill + chunk + buffer rows
    q = gw.make_queries(w, 0, DEV)
    Kb = gw.make_keys(w, w.n_b, 2, DEV)
    Vb = gw.make_values(w, w.n_b, 2, DEV)
    out_g = host(gc.decode_attn(q, Kb, Vb, n_buf)[b_sel:b_sel + 1])[:, qheads]
    oc.decode_attn(np.ascontiguousarray(host(q[b_sel:b_sel + 1])[:, qheads]),
                   np.ascontiguousarray(host(Kb[b_sel:b_sel + 1])[:, heads]),
                   np.ascontiguousarray(host(Vb[b_sel:b_sel + 1])[:, heads]), n_buf)
    rep["attn_vs_f64"], rep["attn_bar_used"] = pu.check_attention(out_g, oc.last_attn_f64)
    say("  ->", rep)
    return rep


def test_config1_llama2_7b():
    run_full(gw.CONFIGS[1], b_sel=9, heads=None, n_buf=7)


def test_config2_llama2_13b():
    run_full(gw.CONFIGS[2], b_sel=17, heads=None, n_buf=20)


def test_config3_long_context():
    run_full(gw.CONFIGS[3], b_sel=0, heads=[0, 13, 31], n_buf=33)


def test_config4_llama3_gqa():
    run_full(gw.CONFIGS[4], b_sel=40, heads=None, n_buf=11)


def test_config4_gear_l():
    run_full(gw.CONFIGS[5], b_sel=3, heads=None, n_buf=1)
