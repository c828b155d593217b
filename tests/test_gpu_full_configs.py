"""GPU parity at the benchmark's full sizes (configs 1-4 and the GEAR-L variant
of config 4), in the launch configuration bench.py times.  The whole batch runs
on the GPU; the oracle recomputes two sampled batch elements (a subset of heads of the one batch element
of the long-context config) from the same bytes, which is exact: Keys are
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


def run_full(w, b_sels, heads, n_buf):
    """b_sels: the batch elements the oracle recomputes (each one whole: the oracle cache holds them
    as its batch)."""
    say("full-size case", w.name, "sampled batch elements", b_sels, "heads", heads, "iters", w.iters)
    H = w.H_kv
    heads = list(range(H)) if heads is None else heads
    gq = w.H_q // H
    qheads = [h * gq + i for h in heads for i in range(gq)]
    nb = len(b_sels)
    cfg = gb.make_config(w.B, H, w.H_q, w.bits, w.group, w.outlier_ppm, w.n_b, w.n, 2, max(w.rank, w.rank_chunk))
    gc = gb.GearCache(cfg, DEV)
    oc = go.OracleCache(nb, len(heads), len(qheads), 128, w.bits, w.group, w.outlier_ppm)
    pick = lambda t: host(t[b_sels])                 # [nb, ...] host copy of the sampled batch elements

    def both(K, V, rank, ib):
        gc.compress(K, V, rank, w.iters, ib)
        Kb, Vb = pick(K), pick(V)
        v_mask = go.filter_values(Vb, w.outlier_ppm)[:, heads] if w.outlier_ppm > 0 else None
        oc.compress(np.ascontiguousarray(Kb[:, heads]), np.ascontiguousarray(Vb[:, heads]), rank, w.iters,
                    np.ascontiguousarray(host(ib[:, b_sels])[:, :, heads]), v_mask)

    K = gw.make_keys(w, w.n, 0, DEV)
    V = gw.make_values(w, w.n, 0, DEV)
    both(K, V, w.rank, gw.make_init_B(w, w.rank, 0, DEV))
    del K, V
    Kc = gw.make_keys(w, w.n_b, 1, DEV)
    Vc = gw.make_values(w, w.n_b, 1, DEV)
    both(Kc, Vc, w.rank_chunk, gw.make_init_B(w, w.rank_chunk, 1, DEV))

    rep = {}
    sl = lambda t: pick(t)[:, heads]
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
        # the low-rank product A B^T of the prefill segment
        A, Bf = [sl(x).astype(np.float64) for x in gc.export_lowrank(which, 0)]
        Lg = np.einsum("bhnr,bhdr->bhnd", A, Bf)
        Lo = np.einsum("bhnr,bhdr->bhnd", segs[0].A.astype(np.float64), segs[0].Bf.astype(np.float64))
        rep[name + "_L_rel"] = float(np.linalg.norm(Lg - Lo) / np.linalg.norm(Lo))
        assert rep[name + "_L_rel"] <= pu.LOWRANK_REL_TOL, rep
        del A, Bf, Lg, Lo
    Kg, Vg = gc.decompress()
    Ko, Vo = oc.decompress()
    rep["K_rel_frob"], rep["V_rel_frob"] = pu.rel_frob(sl(Kg), Ko), pu.rel_frob(sl(Vg), Vo)
    assert rep["K_rel_frob"] <= pu.REL_FROB_TOL and rep["V_rel_frob"] <= pu.REL_FROB_TOL, rep
    del Kg, Vg
    # invariants that hold at any size, checked on the whole batch: exact outlier counts per vector,
    # and the coordinate form of S agrees with its dense form
    if w.outlier_ppm > 0:
        mk, _ = gc.export_sparse(0)
        kv_n = go.outlier_counts(w.n, w.outlier_ppm)[0]
        kv_c = go.outlier_counts(w.n_b, w.outlier_ppm)[0]
        assert (mk[:, :, :w.n].sum(dim=2) == kv_n).all() and (mk[:, :, w.n:].sum(dim=2) == kv_c).all()
        lin, _ = gc.export_sparse_coo(0)
        assert torch.equal(lin, torch.nonzero(mk.reshape(-1)).reshape(-1))
        del mk, lin
        mv, _ = gc.export_sparse(1)
        assert (mv.sum(dim=(1, 3)) == go.outlier_counts(H * 128, w.outlier_ppm)[0]).all()
        del mv
    # decode attention over prefill + chunk + buffer rows
    q = gw.make_queries(w, 0, DEV)
    Kb = gw.make_keys(w, w.n_b, 2, DEV)
    Vb = gw.make_values(w, w.n_b, 2, DEV)
    out_g = pick(gc.decode_attn(q, Kb, Vb, n_buf))[:, qheads]
    oc.decode_attn(np.ascontiguousarray(pick(q)[:, qheads]), np.ascontiguousarray(pick(Kb)[:, heads]),
                   np.ascontiguousarray(pick(Vb)[:, heads]), n_buf)
    rep["attn_vs_f64"], rep["attn_bar_used"] = pu.check_attention(out_g, oc.last_attn_f64)
    say("  ->", rep)
    return rep


def test_config1_llama2_7b():
    run_full(gw.CONFIGS[1], b_sels=[9, 0], heads=None, n_buf=7)


def test_config1_single_round():
    """L = 1 at full size: the only round of Algorithm 2 is also its last."""
    import dataclasses
    run_full(dataclasses.replace(gw.CONFIGS[1], iters=1), b_sels=[5], heads=None, n_buf=20)


def test_config2_llama2_13b():
    run_full(gw.CONFIGS[2], b_sels=[17, 31], heads=None, n_buf=20)


def test_config3_long_context():
    run_full(gw.CONFIGS[3], b_sels=[0], heads=[0, 13, 31], n_buf=33)


def test_config4_llama3_gqa():
    run_full(gw.CONFIGS[4], b_sels=[40, 63], heads=None, n_buf=11)


def test_config4_gear_l():
    run_full(gw.CONFIGS[5], b_sels=[3, 22], heads=None, n_buf=1)
