"""Pins for the oracle's Filter (Eq. 4), Quant (Eq. 2 / Eq. 5) and the packed view.

Each check compares the oracle with something other than itself: a brute-force
sort, hand-computed fixtures, the closed-form error bound of uniform
quantization, or an invariant the definition implies.
"""
import json
import os

import numpy as np
import pytest

from oracle import gear_oracle as go

GOLD = os.path.join(os.path.dirname(__file__), "golden")
F16 = np.float16


# ---------------------------------------------------------------- Filter
def brute_filter(vec, k_top, k_bot):
    """Literal reading of Eq. 4 on one vector with python's sort."""
    vals = [float(x) for x in vec]
    idx = list(range(len(vals)))
    top = sorted(idx, key=lambda i: (-vals[i], i))[:k_top]
    rest = [i for i in idx if i not in set(top)]
    bot = sorted(rest, key=lambda i: (vals[i], i))[:k_bot]
    return set(top), set(bot)


@pytest.mark.parametrize("n,ppm", [(1, 20000), (2, 20000), (3, 500000), (20, 20000), (64, 20000),
                                   (100, 100000), (257, 20000), (512, 20000), (50, 1000000)])
def test_filter_vectors_vs_bruteforce(n, ppm):
    rng = np.random.default_rng(n * 7 + ppm)
    k, kt, kb = go.outlier_counts(n, ppm)
    assert k == -(-ppm * n // 10**6) or k == n
    assert kt + kb == k and kt - kb in (0, 1)
    cases = [
        rng.standard_normal((6, n)),
        np.round(rng.standard_normal((6, n)) * 2) / 2,        # heavy ties
        np.zeros((2, n)),                                     # all equal
        np.where(rng.random((4, n)) < 0.5, 0.0, -0.0),        # +-0 only
        np.round(rng.standard_normal((4, n))) * 0.0 + rng.integers(-1, 2, (4, n)),
    ]
    for c in cases:
        v = c.astype(F16)
        top, bot = go.filter_vectors(v, kt, kb)
        for r in range(v.shape[0]):
            bt, bb = brute_filter(v[r], kt, kb)
            assert set(np.flatnonzero(top[r])) == bt
            assert set(np.flatnonzero(bot[r])) == bb
            assert not (top[r] & bot[r]).any()
            assert top[r].sum() + bot[r].sum() == k


def test_filter_signed_zero_is_one_value():
    v = np.array([[0.0, -0.0, 0.0, -0.0, -1.0, 1.0]], F16)
    top, bot = go.filter_vectors(v, 2, 2)
    assert list(np.flatnonzero(top[0])) == [0, 5]      # 1.0 then the first zero by index
    assert list(np.flatnonzero(bot[0])) == [1, 4]      # -1.0 then the next zero by index


def test_filter_keys_is_per_channel_over_tokens():
    rng = np.random.default_rng(3)
    K = rng.standard_normal((2, 3, 50, 8)).astype(F16)
    K[1, 2, 17, 5] = 100.0
    K[0, 1, 3, 0] = -100.0
    m = go.filter_keys(K, 40000)                      # ceil(0.04*50) = 2 -> 1 top, 1 bottom
    assert m.sum(axis=2).min() == 2 and m.sum(axis=2).max() == 2
    assert m[1, 2, 17, 5] and m[0, 1, 3, 0]
    for b, h, c in [(0, 0, 0), (1, 2, 5), (0, 1, 0)]:
        col = K[b, h, :, c].astype(np.float64)
        assert m[b, h, np.argmax(col), c] and m[b, h, np.argmin(col), c]


def test_filter_values_is_per_token_across_heads():
    rng = np.random.default_rng(4)
    V = rng.standard_normal((2, 4, 6, 16)).astype(F16)      # vector length 64
    V[0, 3, 2, 7] = 50.0
    V[0, 0, 2, 1] = -50.0
    m = go.filter_values(V, 40000)                    # ceil(2.56) = 3 -> 2 top, 1 bottom
    per_token = m.transpose(0, 2, 1, 3).reshape(2, 6, 64).sum(-1)
    assert (per_token == 3).all()
    assert m[0, 3, 2, 7] and m[0, 0, 2, 1]
    # the count is per token across heads, not per head
    assert m[0, :, 2, :].sum() == 3


def test_filter_tie_break_uses_flat_head_channel_index_for_values():
    V = np.zeros((1, 2, 1, 4), F16)
    V[0, :, 0, :] = 1.0                               # 8 equal entries, k = 2 top + 2 bottom
    m = go.filter_values(V, 500000)                   # ceil(0.5*8)=4
    assert list(np.flatnonzero(m.reshape(-1))) == [0, 1, 2, 3]


# ---------------------------------------------------------------- Quant
def test_quant_golden_examples():
    cases = json.load(open(os.path.join(GOLD, "quant_eq2_example.json")))["cases"]
    for c in cases:
        x = np.array(c["x"], F16)[None, :]
        code, s, z, ties = go.quantize(x, c["bits"])
        assert list(code[0]) == c["codes"]
        assert float(s[0]) == c["scale"] and float(z[0]) == c["zero"]
        assert ties == c["ties"]
        deq = code[0].astype(np.float64) * float(s[0]) + float(z[0])
        assert list(deq) == c["dequant"]


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("glen", [1, 5, 20, 64, 128])
def test_quant_error_bound_and_endpoints(bits, glen):
    rng = np.random.default_rng(bits * 100 + glen)
    for scale in (1e-3, 1.0, 37.0):
        y = (rng.standard_t(4, (200, glen)) * scale).astype(F16)
        code, s, z, _ = go.quantize(y, bits)
        qmax = 2 ** bits - 1
        assert code.max() <= qmax
        y64 = y.astype(np.float64)
        d = s.astype(np.float64)
        mn = y64.min(-1)
        assert np.array_equal(z.astype(np.float64), mn)                 # zero-point = group minimum
        d32 = (y64.max(-1) - mn) / qmax
        deq = code * d[:, None] + mn[:, None]
        # Eq. 2: |y - D| <= delta/2 for an exact delta; the fp16-rounded delta
        # moves the top level by at most qmax*|delta - delta32|.
        bound = d / 2 * (1 + 2.0 ** -9) + qmax * np.abs(d - d32) + 1e-12
        assert (np.abs(y64 - deq) <= bound[:, None]).all()
        arg_mn = y64.argmin(-1)
        arg_mx = y64.argmax(-1)
        rows = np.arange(y.shape[0])
        assert (code[rows, arg_mn] == 0).all()
        nz = d > 0
        assert (code[rows, arg_mx][nz] == qmax).all()
        assert np.array_equal(deq[rows, arg_mn], mn)


@pytest.mark.parametrize("bits", [2, 4])
def test_quant_lossless_on_grid_and_idempotent(bits):
    rng = np.random.default_rng(11 + bits)
    qmax = 2 ** bits - 1
    k = rng.integers(0, qmax + 1, (50, 64))
    k[:, 0] = 0
    k[:, 1] = qmax                                    # the group spans the whole code range
    for delta, zero in [(0.5, -3.0), (2.0, 0.0), (0.125, 1.0)]:
        y = (zero + k * delta).astype(F16)
        code, s, z, _ = go.quantize(y, bits)
        assert np.array_equal(code, k.astype(np.uint8))
        assert (s.astype(np.float64) == delta).all() and (z.astype(np.float64) == zero).all()
    # idempotence on arbitrary data: quantizing the (fp32) dequantized values
    # reproduces codes, scale and zero-point
    y = rng.standard_normal((100, 64)).astype(F16)
    code, s, z, _ = go.quantize(y, bits)
    deq32 = code.astype(np.float32) * s.astype(np.float32)[:, None] + z.astype(np.float32)[:, None]
    # re-quantize in the same fp32 arithmetic (dequantized values need not be fp16)
    mn = deq32.min(-1)
    mx = deq32.max(-1)
    full = code.max(-1) == qmax
    d32 = ((mx - mn) / np.float32(qmax)).astype(F16).astype(np.float32)
    assert np.array_equal(mn, z.astype(np.float32))
    assert np.array_equal(d32[full], s.astype(np.float32)[full])
    inv = np.float32(1) / s.astype(np.float32)
    code2 = np.clip(np.rint((deq32 - mn[:, None]) * inv[:, None]), 0, qmax).astype(np.uint8)
    assert np.array_equal(code2, code)


@pytest.mark.parametrize("bits", [2, 4])
def test_quant_codes_agree_with_float64_evaluation_off_ties(bits):
    rng = np.random.default_rng(5)
    y = (rng.standard_normal((500, 64)) * 3).astype(F16)
    code, s, z, _ = go.quantize(y, bits)
    t = (y.astype(np.float64) - z.astype(np.float64)[:, None]) / s.astype(np.float64)[:, None]
    far = np.abs(t - np.floor(t) - 0.5) > 1e-4
    ref = np.clip(np.floor(t + 0.5), 0, 2 ** bits - 1)
    assert np.array_equal(code[far], ref[far].astype(np.uint8))
    assert far.mean() > 0.99


def test_quant_key_and_value_grouping_axes():
    rng = np.random.default_rng(6)
    X = rng.standard_normal((1, 2, 150, 128)).astype(F16)
    # Keys: group = g consecutive tokens of one channel, short last group
    ck, sk, zk, _ = go.quantize_keys(X, 4, 64)
    assert sk.shape == (1, 2, 3, 128)
    for (h, gi, c) in [(0, 0, 0), (1, 1, 77), (1, 2, 127)]:
        grp = X[0, h, gi * 64:(gi + 1) * 64, c].astype(np.float64)
        assert float(zk[0, h, gi, c]) == grp.min()
        assert abs(float(sk[0, h, gi, c]) - (grp.max() - grp.min()) / 15) <= 2.0 ** -11 * float(sk[0, h, gi, c]) + 1e-12
    # Values: group = g consecutive channels of one token
    cv, sv, zv, _ = go.quantize_values(X, 4, 64)
    assert sv.shape == (1, 2, 150, 2)
    for (h, t, gi) in [(0, 0, 0), (1, 149, 1)]:
        grp = X[0, h, t, gi * 64:(gi + 1) * 64].astype(np.float64)
        assert float(zv[0, h, t, gi]) == grp.min()
    # dequant error bound holds through the K/V wrappers too
    dk = go.dequant_keys(ck, sk, zk, 64)
    dv = go.dequant_values(cv, sv, zv, 64)
    assert np.abs(dk - X).max() <= 0.5 * sk.astype(np.float64).max() * 1.01
    assert np.abs(dv - X).max() <= 0.5 * sv.astype(np.float64).max() * 1.01


# ---------------------------------------------------------------- Pack
def test_pack_golden_words_and_roundtrip():
    cases = json.load(open(os.path.join(GOLD, "pack_words.json")))["cases"]
    for c in cases:
        codes = np.array(c["codes"], np.uint8)
        w = go.pack_codes(codes, c["bits"])
        assert [int(x) for x in w] == [int(x, 16) for x in c["words"]]
        assert np.array_equal(go.unpack_codes(w, c["bits"]), codes)
    rng = np.random.default_rng(0)
    for bits in (2, 4):
        codes = rng.integers(0, 2 ** bits, (3, 5, 128)).astype(np.uint8)
        assert np.array_equal(go.unpack_codes(go.pack_codes(codes, bits), bits), codes)


# ---------------------------------------------------------------- byte accounting
def test_kv_size_rows_of_table1():
    spec = json.load(open(os.path.join(GOLD, "kv_size_table1.json")))
    n_all = spec["avg_tokens"]
    for row in spec["rows"]:
        n = n_all - row["n_b"]
        acc = go.compressed_bytes(n, 128, 32, row["bits"], 0 if row["per_vector"] else row["g"], 0, 0)
        total = acc["total"] + 2 * 2 * row["n_b"] * 32 * 128      # + fp16 buffer
        pct = 100.0 * total / (2 * 2 * n_all * 32 * 128)
        assert abs(pct - row["kv_size_pct"]) <= row["tol_pct"], (row["name"], pct)


# ---- the two variants of the follow-up scope: per-head Value Filter, per-vector groups ----
def test_filter_values_per_head_vs_brute_force():
    rng = np.random.default_rng(11)
    B, H, n, d = 2, 3, 5, 128
    V = (rng.integers(-20, 21, size=(B, H, n, d)) * 0.25).astype(np.float16)      # many ties
    V[0, 1, 2, :] = 1.5                                                           # an all-equal vector
    V[1, 0, 0, ::2] = -0.0
    for ppm in (20000, 100000, 500000):
        kv, kt, kb = go.outlier_counts(d, ppm)
        m = go.filter_values(V, ppm, per_head=True)
        assert (m.sum(axis=3) == kv).all()
        for b in range(B):
            for h in range(H):
                for t in range(n):
                    v = [float(x) for x in V[b, h, t]]
                    top = sorted(range(d), key=lambda i: (-v[i], i))[:kt]
                    rest = [i for i in range(d) if i not in top]
                    bot = sorted(rest, key=lambda i: (v[i], i))[:kb]
                    want = np.zeros(d, bool)
                    want[top + bot] = True
                    assert np.array_equal(m[b, h, t], want), (ppm, b, h, t)
    # the two variants rank different vectors: the per-token one couples the heads
    assert not np.array_equal(go.filter_values(V, 20000), go.filter_values(V, 20000, per_head=True))


def test_per_vector_groups_hand_example():
    """Per-vector groups by hand: Keys one group per channel over the call's tokens, Values one
    group per token over both heads.  Values on exact grids, so codes and pairs are known."""
    # Keys: channel 0 runs 0..3 over 4 tokens (scale 1, zero 0), channel 1 is 2 - 0.5 t (scale 0.5, zero 0.5)
    K = np.zeros((1, 1, 4, 2), np.float16)
    K[0, 0, :, 0] = [0, 1, 2, 3]
    K[0, 0, :, 1] = [2.0, 1.5, 1.0, 0.5]
    seg = go.compress_tensor(K, "K", 2, 0, 0, 0, 3, None)
    assert seg.scale.shape == (1, 1, 1, 2) and seg.scale.tolist() == [[[[1.0, 0.5]]]] and seg.zero.tolist() == [[[[0.0, 0.5]]]]
    assert seg.codes[0, 0, :, 0].tolist() == [0, 1, 2, 3] and seg.codes[0, 0, :, 1].tolist() == [3, 2, 1, 0]
    assert np.array_equal(go.reconstruct_segment(seg, 0), K.astype(np.float64))
    # Values: token 0 holds -3..3 over two heads of 2 channels (step 2: scale 2, zero -3), token 1 is constant
    V = np.zeros((1, 2, 2, 2), np.float16)
    V[0, 0, 0] = [-3, 1]
    V[0, 1, 0] = [3, -1]
    V[0, :, 1] = 0.75
    seg = go.compress_tensor(V, "V", 2, 0, 0, 0, 3, None)
    assert seg.scale.shape == (1, 2, 2, 1)
    assert seg.scale[0, :, 0, 0].tolist() == [2.0, 2.0] and seg.zero[0, :, 0, 0].tolist() == [-3.0, -3.0]
    assert seg.scale[0, :, 1, 0].tolist() == [0.0, 0.0] and seg.zero[0, :, 1, 0].tolist() == [0.75, 0.75]
    assert seg.codes[0, 0, 0].tolist() == [0, 2] and seg.codes[0, 1, 0].tolist() == [3, 1]
    assert np.array_equal(go.reconstruct_segment(seg, 0), V.astype(np.float64))


def test_per_vector_groups_error_bound_and_span():
    """Closed form of Eq. 2 with one group per vector: the scale is (max - min) / (2^b - 1) of the WHOLE
    Key channel / Value token row (taken here directly from the input), and |y - D| <= scale / 2."""
    rng = np.random.default_rng(12)
    B, H, n, d, bits = 2, 3, 70, 128, 4
    for kind in ("K", "V"):
        X = rng.standard_normal((B, H, n, d)).astype(np.float16)
        seg = go.compress_tensor(X, kind, bits, 0, 0, 0, 3, None)
        x = X.astype(np.float64)
        if kind == "K":
            span = x.max(axis=2, keepdims=True) - x.min(axis=2, keepdims=True)            # [B,H,1,d]
            assert seg.scale.shape == (B, H, 1, d)
        else:
            rows = x.transpose(0, 2, 1, 3).reshape(B, n, H * d)
            span = (rows.max(axis=2) - rows.min(axis=2))[:, None, :, None]                # [B,1,n,1]
            assert seg.scale.shape == (B, H, n, 1)
        delta = seg.scale.astype(np.float64)
        assert np.allclose(delta, np.broadcast_to(span / 15, delta.shape), rtol=2 ** -10, atol=0)
        err = np.abs(go.reconstruct_segment(seg, 0) - x)
        assert (err <= np.broadcast_to(delta, err.shape) * (0.5 + 2 ** -9) + 15 * 2 ** -11 * np.broadcast_to(delta, err.shape)).all()
