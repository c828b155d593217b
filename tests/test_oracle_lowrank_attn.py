"""Pins for the oracle's SVDSolver (Algorithm 2 / Eq. 6), the GEAR composite
(Eq. 3, Algorithm 1) and the decode attention read (Eq. 1).

References used: LAPACK's full SVD (Eckart-Young optimum), closed forms for
rank-deficient inputs, invariants of an orthogonal projection, and torch's
library softmax attention in fp64 over the reconstructed rows.
"""
import numpy as np
import pytest
import torch

from oracle import gear_oracle as go

F16 = np.float16


def _gap_matrix(rng, n, d, r, gap=0.5):
    U, _ = np.linalg.qr(rng.standard_normal((n, d)))
    Vt, _ = np.linalg.qr(rng.standard_normal((d, d)))
    s = np.concatenate([np.linspace(10, 8, r), gap * 8 * np.linspace(1.0, 0.1, d - r)])
    return (U * s) @ Vt.T, s


@pytest.mark.parametrize("n,d,r", [(40, 16, 2), (100, 32, 4), (64, 128, 8)])
def test_svdsolver_structure_and_eckart_young_bound(n, d, r):
    rng = np.random.default_rng(n + d + r)
    R = rng.standard_normal((n, d))
    B0 = rng.uniform(-1, 1, (d, r))
    for iters in (1, 2, 3):
        A, Bm = go.svd_solver(R, B0, iters)
        assert np.allclose(A.T @ A, np.eye(r), atol=1e-10)          # A orthonormal
        assert np.allclose(Bm, R.T @ A, atol=1e-10)                  # B = R^T A
        err = np.linalg.norm(R - A @ Bm.T)
        sv = np.linalg.svd(R, compute_uv=False)
        opt = np.sqrt((sv[r:] ** 2).sum())
        assert err >= opt * (1 - 1e-12)                              # Eckart-Young
        assert err <= np.linalg.norm(R) * (1 + 1e-12)                # a projection never adds error


def test_svdsolver_exact_when_rank_at_most_r_any_iters():
    rng = np.random.default_rng(1)
    for r_true, r in [(1, 2), (3, 4), (4, 4)]:
        R = rng.standard_normal((60, r_true)) @ rng.standard_normal((r_true, 32))
        B0 = rng.uniform(-1, 1, (32, r))
        for iters in (1, 2, 3, 5):
            A, Bm = go.svd_solver(R, B0, iters)
            assert np.linalg.norm(R - A @ Bm.T) <= 1e-6 * np.linalg.norm(R)


def test_svdsolver_within_1e3_of_optimum():
    rng = np.random.default_rng(2)
    # spectral gap sigma_{r+1}/sigma_r = 0.25, three rounds (the default)
    R, s = _gap_matrix(rng, 200, 64, 4, gap=0.25)
    opt = np.sqrt((s[4:] ** 2).sum())
    A, Bm = go.svd_solver(R, rng.uniform(-1, 1, (64, 4)), 3)
    assert abs(np.linalg.norm(R - A @ Bm.T) - opt) <= 1e-3 * opt
    # a gap of 0.5 needs one more round for the same accuracy
    R, s = _gap_matrix(rng, 200, 64, 4, gap=0.5)
    opt = np.sqrt((s[4:] ** 2).sum())
    A, Bm = go.svd_solver(R, rng.uniform(-1, 1, (64, 4)), 4)
    assert abs(np.linalg.norm(R - A @ Bm.T) - opt) <= 1e-3 * opt
    # a tiny unstructured matrix (sigma_3/sigma_2 = 0.84), many rounds: converges to the optimum
    rng = np.random.default_rng(2)
    R2 = rng.standard_normal((12, 8))
    sv = np.linalg.svd(R2, compute_uv=False)
    A2, B2 = go.svd_solver(R2, rng.uniform(-1, 1, (8, 2)), 30)
    opt2 = np.sqrt((sv[2:] ** 2).sum())
    assert abs(np.linalg.norm(R2 - A2 @ B2.T) - opt2) <= 1e-3 * opt2


def test_svdsolver_matches_top_singular_subspace_rank1():
    rng = np.random.default_rng(3)
    u = rng.standard_normal(50)
    v = rng.standard_normal(16)
    R = 5.0 * np.outer(u, v) + 1e-3 * rng.standard_normal((50, 16))
    A, Bm = go.svd_solver(R, rng.uniform(-1, 1, (16, 1)), 3)
    U, S, Vt = np.linalg.svd(R, full_matrices=False)
    assert abs(abs(A[:, 0] @ U[:, 0]) - 1) < 1e-6
    assert np.allclose(np.abs(Bm[:, 0]), np.abs(S[0] * Vt[0]), atol=1e-4 * S[0])


def test_svdsolver_independent_of_intermediate_orthonormalisation():
    rng = np.random.default_rng(4)
    R = rng.standard_normal((80, 32))
    B0 = rng.uniform(-1, 1, (32, 4))
    A, Bm = go.svd_solver(R, B0, 3)
    # same algorithm with every intermediate B orthonormalised (span unchanged)
    Bt = B0.copy()
    for l in range(3):
        Bt = np.linalg.qr(Bt)[0]
        At = R @ Bt
        if l == 2:
            At = np.linalg.qr(At)[0]
        Bt = R.T @ At
    assert np.linalg.norm(A @ Bm.T - At @ Bt.T) <= 1e-6 * np.linalg.norm(A @ Bm.T)


def test_orth_zero_column_rule_and_transposed_operand_mistake():
    M = np.zeros((10, 3))
    M[:, 0] = 1.0
    M[:, 1] = 2.0                 # dependent on column 0
    Q = go.orth(M)
    assert np.allclose(Q[:, 0], 1 / np.sqrt(10))
    assert (Q[:, 1] == 0).all() and (Q[:, 2] == 0).all()
    # R^T A, not R A^T or A^T R: shapes and values checked against a direct sum
    rng = np.random.default_rng(5)
    R = rng.standard_normal((7, 5))
    A, Bm = go.svd_solver(R, rng.uniform(-1, 1, (5, 2)), 2)
    ref = np.zeros((5, 2))
    for i in range(7):
        for c in range(5):
            for k in range(2):
                ref[c, k] += R[i, c] * A[i, k]
    assert np.allclose(Bm, ref)


# ---------------------------------------------------------------- composite
def _small_kv(rng, B=1, H=2, n=96, d=128):
    K = rng.standard_normal((B, H, n, d))
    K[:, :, :, 5] *= 15
    V = rng.standard_t(4, (B, H, n, d))
    return K.astype(F16), V.astype(F16)


@pytest.mark.parametrize("bits", [2, 4])
def test_composite_reduces_error_and_components_are_consistent(bits):
    rng = np.random.default_rng(7)
    K, V = _small_kv(rng)
    init = rng.uniform(-1, 1, (2, 1, 2, 128, 4)).astype(np.float32)
    for X, kind, ini in [(K, "K", init[0]), (V, "V", init[1])]:
        full = go.compress_tensor(X, kind, bits, 64, 20000, 4, 3, ini)
        nolr = go.compress_tensor(X, kind, bits, 64, 20000, 0, 3, None)
        plain = go.compress_tensor(X, kind, bits, 64, 0, 0, 3, None)
        X64 = X.astype(np.float64)
        e_full = np.linalg.norm(X64 - go.reconstruct_segment(full, 64))
        e_nolr = np.linalg.norm(X64 - go.reconstruct_segment(nolr, 64))
        e_plain = np.linalg.norm(X64 - go.reconstruct_segment(plain, 64))
        assert e_full <= e_nolr * (1 + 1e-3)          # low-rank term (fp16-rounded factors)
        assert e_nolr < e_plain                       # outlier filtering helps on heavy tails
        # S holds bit-exact copies on its support, zero elsewhere; Y is 0 there
        assert np.array_equal(full.svals[full.mask], X[full.mask])
        assert (full.svals[~full.mask] == 0).all()
        # outlier positions are quantized as the value 0 (Eq. 5 quantizes X - S)
        assert np.array_equal(full.codes, nolr.codes)
        # r = 0 and s = 0 is plain group quantization: error bounded by delta/2
        if kind == "V":
            Dh = go.dequant_values(plain.codes, plain.scale, plain.zero, 64)
            assert np.abs(X64 - Dh).max() <= plain.scale.astype(np.float64).max() * 0.5 * 1.01


def test_composite_lossless_grid_is_bit_exact():
    rng = np.random.default_rng(8)
    k = rng.integers(0, 4, (1, 2, 64, 128))
    k[:, :, 0, :] = 0
    k[:, :, 1, :] = 3
    K = (-1.0 + 0.5 * k).astype(F16)                  # every key group spans codes 0..3
    seg = go.compress_tensor(K, "K", 2, 64, 0, 4, 3, rng.uniform(-1, 1, (1, 2, 128, 4)).astype(np.float32))
    assert np.array_equal(go.reconstruct_segment(seg, 64).astype(F16), K)
    assert (seg.A == 0).all() and (seg.Bf == 0).all()


# ---------------------------------------------------------------- attention
def _cache_with_segments(rng, B=2, H=2, Hq=4, n=70, n_chunk=20):
    oc = go.OracleCache(B, H, Hq, 128, 4, 64, 20000)
    K = rng.standard_normal((B, H, n, 128)).astype(F16)
    V = rng.standard_t(4, (B, H, n, 128)).astype(F16)
    oc.compress(K, V, 4, 3, rng.uniform(-1, 1, (2, B, H, 128, 4)).astype(np.float32))
    K2 = rng.standard_normal((B, H, n_chunk, 128)).astype(F16)
    V2 = rng.standard_t(4, (B, H, n_chunk, 128)).astype(F16)
    oc.compress(K2, V2, 2, 3, rng.uniform(-1, 1, (2, B, H, 128, 2)).astype(np.float32))
    return oc


def test_decode_attn_matches_library_attention_over_reconstructed_rows():
    rng = np.random.default_rng(9)
    oc = _cache_with_segments(rng)
    assert oc.n_total == 90
    q = rng.standard_normal((2, 4, 1, 128)).astype(F16)
    Kb = rng.standard_normal((2, 2, 20, 128)).astype(F16)
    Vb = rng.standard_normal((2, 2, 20, 128)).astype(F16)
    out = oc.decode_attn(q, Kb, Vb, 7)
    Kh, Vh = oc.reconstruct()
    Kall = np.concatenate([Kh, Kb[:, :, :7].astype(np.float64)], 2)
    Vall = np.concatenate([Vh, Vb[:, :, :7].astype(np.float64)], 2)
    tq = torch.from_numpy(q.astype(np.float64))
    tk = torch.from_numpy(np.repeat(Kall, 2, axis=1))     # GQA: 2 query heads per KV head
    tv = torch.from_numpy(np.repeat(Vall, 2, axis=1))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).numpy()
    assert np.abs(out.astype(np.float64) - ref).max() <= 1e-3
    assert np.array_equal(out, ref.astype(F16))


def test_decode_attn_special_cases():
    rng = np.random.default_rng(10)
    oc = _cache_with_segments(rng)
    Kh, Vh = oc.reconstruct()
    # q = 0 -> uniform weights -> mean of the reconstructed value rows
    q0 = np.zeros((2, 4, 1, 128), F16)
    out = oc.decode_attn(q0)
    ref = np.repeat(Vh.mean(axis=2, keepdims=True), 2, axis=1)
    assert np.abs(out.astype(np.float64) - ref).max() <= 2e-3
    # query heads of one GQA group with equal q give equal outputs
    q = rng.standard_normal((2, 4, 1, 128)).astype(F16)
    q[:, 1] = q[:, 0]
    out = oc.decode_attn(q)
    assert np.array_equal(out[:, 0], out[:, 1])
    # buffer only (no compressed segment yet): plain fp16 attention
    empty = go.OracleCache(1, 1, 1, 128, 4, 64, 20000)
    Kb = rng.standard_normal((1, 1, 5, 128)).astype(F16)
    Vb = rng.standard_normal((1, 1, 5, 128)).astype(F16)
    qq = rng.standard_normal((1, 1, 1, 128)).astype(F16)
    o = empty.decode_attn(qq, Kb, Vb, 5)
    s = Kb[0, 0].astype(np.float64) @ qq[0, 0, 0].astype(np.float64) / np.sqrt(128)
    p = np.exp(s - s.max()); p /= p.sum()
    assert np.array_equal(o[0, 0, 0], (p @ Vb[0, 0].astype(np.float64)).astype(F16))
    # one-row cache: output = that row
    one = go.OracleCache(1, 1, 1, 128, 4, 64, 0)
    one.compress(Kb[:, :, :1], Vb[:, :, :1], 0, 3, None)
    o1 = one.decode_attn(qq)
    assert np.array_equal(o1[0, 0, 0], one.reconstruct()[1][0, 0, 0].astype(F16))


def test_decode_attn_on_lossless_grid_equals_fp16_attention():
    rng = np.random.default_rng(12)
    k = rng.integers(0, 16, (1, 2, 64, 128)); k[:, :, 0, :] = 0; k[:, :, 1, :] = 15
    K = (-2.0 + 0.25 * k).astype(F16)
    kv = rng.integers(0, 16, (1, 2, 64, 128)); kv[..., 0] = 0; kv[..., 1] = 15; kv[..., 64] = 0; kv[..., 65] = 15
    V = (-1.0 + 0.125 * kv).astype(F16)
    oc = go.OracleCache(1, 2, 2, 128, 4, 64, 0)
    oc.compress(K, V, 2, 3, rng.uniform(-1, 1, (2, 1, 2, 128, 2)).astype(np.float32))
    q = rng.standard_normal((1, 2, 1, 128)).astype(F16)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q.astype(np.float64)), torch.from_numpy(K.astype(np.float64)),
        torch.from_numpy(V.astype(np.float64))).numpy()
    assert np.array_equal(oc.decode_attn(q), ref.astype(F16))


def test_streaming_segments_are_independent_compress_calls():
    """Each flushed buffer is compressed alone (own groups, own S, own factors):
    segment 1 of a two-segment cache equals a fresh compress of the same tokens."""
    rng = np.random.default_rng(13)
    oc = _cache_with_segments(rng)
    seg = oc.K[1]
    X = go.reconstruct_segment(seg, 64)
    assert seg.n == 20 and seg.scale.shape[2] == 1          # 20 < g: one short group per channel
    assert seg.mask.sum(axis=2).max() == 1                  # ceil(2% of 20) = 1 per channel (top only)
    assert X.shape == (2, 2, 20, 128)


def test_multi_query_read_vs_masked_library_attention():
    """The multi-query read against torch's attention in fp64 with an explicit mask over
    [compressed rows | buffer rows], and its q_len = 1 case against the single-query read."""
    import torch
    rng = np.random.default_rng(21)
    B, H, Hq, n, d, n_buf, q_len = 2, 2, 4, 37, 128, 9, 4
    oc = go.OracleCache(B, H, Hq, d, 4, 64, 20000)
    K = rng.standard_normal((B, H, n, d)).astype(np.float16)
    V = rng.standard_normal((B, H, n, d)).astype(np.float16)
    oc.compress(K, V, 2, 3, rng.uniform(-1, 1, (2, B, H, d, 2)).astype(np.float32))
    Kb = rng.standard_normal((B, H, 12, d)).astype(np.float16)
    Vb = rng.standard_normal((B, H, 12, d)).astype(np.float16)
    q = rng.standard_normal((B, Hq, q_len, d)).astype(np.float16)
    Kh, Vh = oc.reconstruct()
    Kall = torch.from_numpy(np.concatenate([Kh, Kb[:, :, :n_buf].astype(np.float64)], axis=2)).repeat_interleave(2, dim=1)
    Vall = torch.from_numpy(np.concatenate([Vh, Vb[:, :, :n_buf].astype(np.float64)], axis=2)).repeat_interleave(2, dim=1)
    for causal in (True, False):
        got = go.decode_attn_multi(oc, q, Kb, Vb, n_buf, causal)
        mask = torch.ones(q_len, n + n_buf, dtype=torch.bool)
        if causal:
            for j in range(q_len):
                mask[j, n + n_buf - q_len + j + 1:] = False
        want = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q.astype(np.float64)), Kall, Vall,
                                                                attn_mask=mask).numpy()
        assert np.abs(got - want).max() < 1e-12
    oc.decode_attn(q[:, :, :1], Kb, Vb, n_buf)
    assert np.abs(go.decode_attn_multi(oc, q[:, :, :1], Kb, Vb, n_buf, True) - oc.last_attn_f64).max() < 1e-15


def test_low_rank_term_on_the_most_recent_tokens_only():
    """n_lowrank: codes on a lossless grid plus a rank-1 perturbation u v^T over ALL rows that leaves the
    quantizer alone, so the residual is exactly u v^T.  The solver run on the recent rows must recover
    u v^T there (rank 1 <= r is reproduced for any L) and leave the earlier rows without a low-rank term."""
    rng = np.random.default_rng(31)
    n, d, m, step = 96, 128, 40, 2.0 ** -10
    k = rng.integers(1, 3, size=(1, 1, n, d))
    k[:, :, 0::64, :] = 0
    k[:, :, 1::64, :] = 3
    u = rng.integers(-7, 8, size=(1, 1, n, 1)).astype(np.float64)
    u[:, :, 0::64] = 0
    u[:, :, 1::64] = 0
    v = rng.integers(1, 3, size=(1, 1, 1, d)) * step
    X = (-1.0 + 0.5 * k + u * v).astype(np.float16)
    assert np.array_equal(X.astype(np.float64), -1.0 + 0.5 * k + u * v)
    B0 = rng.uniform(-1, 1, (1, 1, d, 3)).astype(np.float32)
    seg = go.compress_tensor(X, "K", 2, 64, 0, 3, 2, B0, n_lowrank=m)
    L = np.einsum("bhnr,bhdr->bhnd", seg.A.astype(np.float64), seg.Bf.astype(np.float64))
    assert not seg.A[:, :, :n - m].any() and np.abs(L[:, :, :n - m]).max() == 0.0
    assert np.abs(L[:, :, n - m:] - (u * v)[:, :, n - m:]).max() <= 2e-3 * 14 * step
    Xh = go.reconstruct_segment(seg, 64)
    assert np.abs(Xh[:, :, :n - m] - (-1.0 + 0.5 * k[:, :, :n - m])).max() == 0.0       # Filter + Quant only
    # n_lowrank = n is the plain call, n_lowrank = 0 has no low-rank term at all
    full = go.compress_tensor(X, "K", 2, 64, 0, 3, 2, B0, n_lowrank=n)
    plain = go.compress_tensor(X, "K", 2, 64, 0, 3, 2, B0)
    assert np.array_equal(full.A, plain.A) and np.array_equal(full.Bf, plain.Bf)
    assert not go.compress_tensor(X, "K", 2, 64, 0, 3, 2, B0, n_lowrank=0).A.any()
