"""The approximation-error study (paper_2403_05527_amd/error_study.py) on a small workload: its
numbers must agree with the same quantities computed from the CPU oracle's reconstruction, and
show the ordering the method is built on (each error-reduction term lowers the error)."""
import dataclasses

import numpy as np
import pytest
import torch

import gear_workloads as gw
from oracle import gear_oracle as go
from paper_2403_05527_amd import error_study as es

pytestmark = pytest.mark.gpu


def test_error_study_matches_oracle_and_orders_the_methods():
    w = gw.Workload("study", B=1, H_kv=4, H_q=4, n=384, bits=2, group=64, outlier_ppm=20000, rank=4, rank_chunk=2,
                    n_b=20, steps=1, seed=33)
    rep = es.study(w, spectrum_heads=2)
    rows = {r["method"]: r for r in rep["methods"]}
    K = gw.make_keys(w, w.n, 0, "cuda:0").cpu().numpy()
    V = gw.make_values(w, w.n, 0, "cuda:0").cpu().numpy()
    ib = gw.make_init_B(w, 4, 0, "cuda:0").cpu().numpy()
    for name, use_s, use_l in es.METHODS:
        oc = go.OracleCache(1, 4, 4, 128, 2, 64, w.outlier_ppm if use_s else 0)
        oc.compress(K, V, w.rank if use_l else 0, 3, ib)
        Kh, Vh = oc.decompress()
        for t, X, Xh in (("K", K, Kh), ("V", V, Vh)):
            want = np.linalg.norm(Xh.astype(np.float64) - X.astype(np.float64)) / np.linalg.norm(X.astype(np.float64))
            assert abs(rows[name][t + "_rel_frob"] - want) <= 1e-3 * want + 1e-6, (name, t)
    for t in ("K_rel_frob", "V_rel_frob"):
        assert rows["GEAR"][t] < rows["quant+S"][t] < rows["quant"][t]
        assert rows["GEAR"][t] < rows["quant+L"][t] < rows["quant"][t]
    assert rows["GEAR"]["kv_size_fraction"] > rows["quant"]["kv_size_fraction"]
    # the residual's leading direction carries more than 1/128 of its energy, the top 4 less than all of it
    for v in rep["spectrum"].values():
        assert 1.0 / 128 < v["energy_in_top_r"]["1"] < v["energy_in_top_r"]["4"] < 1.0
        assert v["sigma_over_sigma1"][0] == 1.0
