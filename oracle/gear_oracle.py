"""CPU oracle for GEAR KV-cache compression and the compressed-cache attention read.

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, step-by-step statement
of what the hot path computes, written from the paper (GEAR, arXiv 2403.05527).
Only tests, the smoke check and the benchmark's cpu_baseline leg may import it;
the product (the HIP library and its Python binding) never does, and the two
share no code.

GEAR is an encoding, not a faster route to an exact result, so the oracle takes
the paper's steps in the paper's order (Algorithm 1 with Eq. 2, 4, 5, 6 and
Algorithm 2).  numpy is used for vectorised elementwise work, sorting and
matmul; there is no blocking, fusion or reordering beyond what the paper states.

Precision.  The paper fixes none for the quantizer arithmetic; integer codes are
decided in IEEE fp32 with the operation sequence written in `quantize` (the
kernel's precision, so that both sides take the rounding decision in the same
arithmetic).  Everything that is not an integer decision (residual, power
iteration, reconstruction, attention) is computed in fp64 from the *stored*
fp16 quantities.

Parity pins (tests/test_oracle_*.py): Filter vs brute-force sort (also the
per-head Value variant); the per-vector grouping vs a hand-computed example and
Table 1's KCVT KV-size row; Quant vs the
closed-form error bound of Eq. 2, end-point codes, idempotence and a lossless
grid; pack vs hand-computed words; SVDSolver vs a full LAPACK SVD (Eckart-Young
bound, exactness for rank <= r, orthonormality); composite monotonicity;
attention vs a library softmax attention over the reconstructed rows.
The absolute error level GEAR reaches on real model KV caches (Fig. 1a / 2a) is
"parity unpinned": it needs real activations.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

F16 = np.float16
F32 = np.float32
F64 = np.float64


# --------------------------------------------------------------------------
# Filter_s  (Eq. 4)
# --------------------------------------------------------------------------
def outlier_counts(n_v: int, outlier_ppm: int):
    """How many entries of a length-n_v vector Filter_s keeps (Eq. 4: "s/2 % of
    maximum and minimum entries of each vector").  Total = ceil(s * n_v) in
    integer arithmetic, the top side takes the odd one."""
    k = -((-outlier_ppm * n_v) // 1_000_000)
    k = max(0, min(k, n_v))
    return k, (k + 1) // 2, k // 2


def filter_vectors(v16: np.ndarray, k_top: int, k_bot: int):
    """v16: fp16 [M, N], one vector per row.  Returns boolean masks (top, bot).

    top = first k_top entries in the order (value descending, index ascending);
    bot = first k_bot of the remaining entries in (value ascending, index
    ascending).  Values compare numerically (-0 == +0)."""
    v = v16.astype(F64)                      # exact
    top = np.zeros(v.shape, dtype=bool)
    bot = np.zeros(v.shape, dtype=bool)
    if k_top > 0:
        order = np.argsort(-v, axis=1, kind="stable")
        np.put_along_axis(top, order[:, :k_top], True, axis=1)
    if k_bot > 0:
        rest = np.where(top, np.inf, v)      # entries already taken go last
        order = np.argsort(rest, axis=1, kind="stable")
        np.put_along_axis(bot, order[:, :k_bot], True, axis=1)
    return top, bot


def filter_keys(K16: np.ndarray, outlier_ppm: int) -> np.ndarray:
    """Eq. 4, X = K: the vector is one channel of one head over the n tokens of
    this call.  K16: fp16 [B, H, n, d].  Returns the support of S as a mask."""
    B, H, n, d = K16.shape
    _, kt, kb = outlier_counts(n, outlier_ppm)
    vec = np.ascontiguousarray(K16.transpose(0, 1, 3, 2)).reshape(B * H * d, n)
    top, bot = filter_vectors(vec, kt, kb)
    m = (top | bot).reshape(B, H, d, n).transpose(0, 1, 3, 2)
    return np.ascontiguousarray(m)


def filter_values(V16: np.ndarray, outlier_ppm: int, per_head: bool = False) -> np.ndarray:
    """Eq. 4, X = V: the vector is one token's row over all heads' channels,
    X in R^{n x d} with d = H*d_H (Sec. 2 notation); index j = h*d_H + c.
    per_head: the variant that ranks each head's d_H channels of a token on their
    own (the vector is X_h[t, :], index c), which keeps every head independent."""
    B, H, n, d = V16.shape
    if per_head:
        _, kt, kb = outlier_counts(d, outlier_ppm)
        top, bot = filter_vectors(V16.reshape(B * H * n, d), kt, kb)
        return (top | bot).reshape(B, H, n, d)
    _, kt, kb = outlier_counts(H * d, outlier_ppm)
    vec = np.ascontiguousarray(V16.transpose(0, 2, 1, 3)).reshape(B * n, H * d)
    top, bot = filter_vectors(vec, kt, kb)
    m = (top | bot).reshape(B, n, H, d).transpose(0, 2, 1, 3)
    return np.ascontiguousarray(m)


# --------------------------------------------------------------------------
# Quant_b  (Eq. 2 applied as Eq. 5 to Y = X - S)
# --------------------------------------------------------------------------
def quantize(y16: np.ndarray, bits: int):
    """Uniform asymmetric quantization of groups (Eq. 2).  y16: fp16 [..., L],
    one group per trailing row.  Returns (codes u8 [..., L], scale fp16 [...],
    zero fp16 [...], n_ties).

    fp32 sequence (each op rounded to nearest even, no fused multiply-add):
      mn, mx        = min, max of the group
      delta32       = (mx - mn) / (2^b - 1)
      delta         = fp16(delta32)          <- stored, and used from here on
      inv           = 1 / fp32(delta)
      t             = (y - mn) * inv
      code          = clamp(round_half_even(t), 0, 2^b - 1);  all 0 if delta == 0
    """
    qmax = F32(2 ** bits - 1)
    y = y16.astype(F32)
    mn = y.min(axis=-1) + F32(0)             # +0 turns a -0 minimum into +0
    mx = y.max(axis=-1) + F32(0)
    delta32 = (mx - mn) / qmax
    delta16 = delta32.astype(F16)
    delta = delta16.astype(F32)
    safe = np.where(delta > 0, delta, F32(1))
    inv = F32(1) / safe
    t = (y - mn[..., None]) * inv[..., None]
    r = np.rint(t)                           # ties to even
    code = np.clip(r, F32(0), qmax)
    code = np.where(delta[..., None] > 0, code, F32(0)).astype(np.uint8)
    ties = int(np.count_nonzero((np.abs(t - np.floor(t) - F32(0.5)) == 0) & (delta[..., None] > 0)))
    return code, delta16, mn.astype(F16), ties


def quantize_keys(Y16: np.ndarray, bits: int, g: int):
    """Per-channel grouping along tokens (KIVI-style Key grouping): a group is g
    consecutive tokens of one channel, counted from token 0 of the call; the
    last group is short when g does not divide n.
    Returns codes [B,H,n,d], scale/zero fp16 [B,H,ceil(n/g),d], ties."""
    B, H, n, d = Y16.shape
    ng = (n + g - 1) // g
    codes = np.zeros((B, H, n, d), np.uint8)
    scale = np.zeros((B, H, ng, d), F16)
    zero = np.zeros((B, H, ng, d), F16)
    ties = 0
    for gi in range(ng):
        t0, t1 = gi * g, min(n, (gi + 1) * g)
        blk = Y16[:, :, t0:t1, :].transpose(0, 1, 3, 2)          # [..., d, len]
        c, s, z, tt = quantize(blk, bits)
        codes[:, :, t0:t1, :] = c.transpose(0, 1, 3, 2)
        scale[:, :, gi, :] = s
        zero[:, :, gi, :] = z
        ties += tt
    return codes, scale, zero, ties


def quantize_values(Y16: np.ndarray, bits: int, g: int):
    """Per-token grouping along channels: a group is g consecutive channels of
    one token inside one head (g divides d_H).
    Returns codes [B,H,n,d], scale/zero fp16 [B,H,n,d/g], ties."""
    B, H, n, d = Y16.shape
    assert d % g == 0
    c, s, z, ties = quantize(Y16.reshape(B, H, n, d // g, g), bits)
    return c.reshape(B, H, n, d), s, z, ties


def quantize_values_whole_token(Y16: np.ndarray, bits: int):
    """The coarse per-vector grouping of the background section ("KCVT"): all Value
    entries of one token, over every head, form one group of size d = H * d_H.
    Returns codes [B,H,n,d_H] and scale/zero fp16 [B,H,n,1] (each head carries its
    token's pair, so the views have the shape of a per-head grouping with g = d_H)."""
    B, H, n, d = Y16.shape
    rows = np.ascontiguousarray(Y16.transpose(0, 2, 1, 3)).reshape(B, n, H * d)
    c, s, z, ties = quantize(rows, bits)
    codes = np.ascontiguousarray(c.reshape(B, n, H, d).transpose(0, 2, 1, 3))
    scale = np.ascontiguousarray(np.broadcast_to(s[:, None, :, None], (B, H, n, 1)))
    zero = np.ascontiguousarray(np.broadcast_to(z[:, None, :, None], (B, H, n, 1)))
    return codes, scale, zero, ties


def dequant_keys(codes, scale, zero, g):
    """D-hat for Keys in fp64 from the stored codes / fp16 scale / fp16 zero."""
    n = codes.shape[2]
    s = np.repeat(scale.astype(F64), g, axis=2)[:, :, :n, :]
    z = np.repeat(zero.astype(F64), g, axis=2)[:, :, :n, :]
    return codes.astype(F64) * s + z


def dequant_values(codes, scale, zero, g):
    s = np.repeat(scale.astype(F64), g, axis=3)
    z = np.repeat(zero.astype(F64), g, axis=3)
    return codes.astype(F64) * s + z


def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """Canonical packed view: the codes of one token row are consecutive along
    d_H, little-endian inside 32-bit words (channel c sits at bit
    (c mod 32/b)*b of word floor(c*b/32)).  codes u8 [..., d] -> u32 [..., d*b/32]."""
    per = 32 // bits
    d = codes.shape[-1]
    assert d % per == 0
    c = codes.astype(np.uint64).reshape(codes.shape[:-1] + (d // per, per))
    shifts = (np.arange(per, dtype=np.uint64) * np.uint64(bits))
    return (c << shifts).sum(axis=-1).astype(np.uint32)


def unpack_codes(words: np.ndarray, bits: int) -> np.ndarray:
    per = 32 // bits
    shifts = (np.arange(per, dtype=np.uint32) * np.uint32(bits))
    c = (words[..., None] >> shifts) & np.uint32(2 ** bits - 1)
    return c.reshape(words.shape[:-1] + (words.shape[-1] * per,)).astype(np.uint8)


# --------------------------------------------------------------------------
# SVDSolver_r  (Algorithm 2, power iteration)
# --------------------------------------------------------------------------
def orth(M: np.ndarray) -> np.ndarray:
    """Q factor of a thin QR of M [m, r] (the algorithm's QRdecomposition step)
    by modified Gram-Schmidt applied twice, fp64.  A column that is exactly 0,
    or whose norm after projection falls below 1e-12 of its norm before, is
    set to 0 (rank-deficient input)."""
    Q = np.array(M, dtype=F64, copy=True)
    m, r = Q.shape
    for j in range(r):
        before = np.linalg.norm(Q[:, j])
        if before == 0.0:
            Q[:, j] = 0.0
            continue
        for _ in range(2):
            for i in range(j):
                Q[:, j] -= (Q[:, i] @ Q[:, j]) * Q[:, i]
        after = np.linalg.norm(Q[:, j])
        if after <= 1e-12 * before:
            Q[:, j] = 0.0
        else:
            Q[:, j] /= after
    return Q


def svd_solver(R: np.ndarray, B0: np.ndarray, iters: int):
    """Algorithm 2 on one head's residual R [n, d_H] with start B0 [d_H, r]:
    `iters` rounds of A = R B, B = R^T A, with B then A replaced by the Q factor
    of their QR in the last round only.  (A's own random start is overwritten
    before use, so only B's start matters.)  Returns fp64 (A [n,r], B [d_H,r])."""
    R = R.astype(F64)
    Bm = B0.astype(F64)
    A = np.zeros((R.shape[0], Bm.shape[1]), F64)
    for l in range(iters):
        last = (l == iters - 1)
        if last:
            Bm = orth(Bm)
        A = R @ Bm
        if last:
            A = orth(A)
        Bm = R.T @ A
    return A, Bm


# --------------------------------------------------------------------------
# One compressed segment, and the cache (Algorithm 1)
# --------------------------------------------------------------------------
@dataclass
class Segment:
    """What one `compress` call stores for one tensor (K or V)."""
    kind: str                 # "K" or "V"
    n: int
    codes: np.ndarray         # u8  [B,H,n,d]
    scale: np.ndarray         # f16 [B,H,ng,d] (K) / [B,H,n,d/g] (V)
    zero: np.ndarray          # f16 same shape
    mask: np.ndarray          # bool [B,H,n,d]  support of S
    svals: np.ndarray         # f16 [B,H,n,d]   S (0 off the support)
    A: np.ndarray             # f16 [B,H,n,r]
    Bf: np.ndarray            # f16 [B,H,d,r]
    ties: int = 0


def compress_tensor(X16: np.ndarray, kind: str, bits: int, g: int, outlier_ppm: int,
                    rank: int, iters: int, init_B: Optional[np.ndarray],
                    mask: Optional[np.ndarray] = None, v_per_head: bool = False,
                    n_lowrank: Optional[int] = None) -> Segment:
    """Algorithm 1, prefill-phase body for one tensor X in {K, V} (the decoding
    phase runs the same body on the buffered tokens):
      S = Filter_s(X); D-hat = Quant_b(X - S); R = X - D-hat - S;
      L_h = SVDSolver_r(R_h) for every head (and batch element).
    g = 0 selects the coarse per-vector grouping (one group per Key channel of the
    call, one per Value token over all heads).  n_lowrank: the ablation of Sec. 4.3 that
    applies the low-rank approximation to the n_lowrank most recent tokens only
    (SVDSolver on their residual rows; the earlier tokens get no low-rank term)."""
    assert X16.dtype == F16
    B, H, n, d = X16.shape
    if mask is None:       # a caller that holds only some heads passes the support it computed on all
        if outlier_ppm <= 0:
            mask = np.zeros(X16.shape, bool)
        elif kind == "K":
            mask = filter_keys(X16, outlier_ppm)
        else:
            mask = filter_values(X16, outlier_ppm, v_per_head)
    svals = np.where(mask, X16, F16(0))
    Y16 = np.where(mask, F16(0), X16)                       # X - S, exact
    if kind == "K":
        gk = n if g == 0 else g
        codes, scale, zero, ties = quantize_keys(Y16, bits, gk)
        Dh = dequant_keys(codes, scale, zero, gk)
    elif g == 0:
        codes, scale, zero, ties = quantize_values_whole_token(Y16, bits)
        Dh = dequant_values(codes, scale, zero, d)
    else:
        codes, scale, zero, ties = quantize_values(Y16, bits, g)
        Dh = dequant_values(codes, scale, zero, g)
    R = Y16.astype(F64) - Dh                                # = X - D-hat - S
    A16 = np.zeros((B, H, n, rank), F16)
    B16 = np.zeros((B, H, d, rank), F16)
    first = 0 if n_lowrank is None else n - n_lowrank
    if rank > 0 and first < n:
        for b in range(B):
            for h in range(H):
                A, Bm = svd_solver(R[b, h, first:], init_B[b, h], iters)
                A16[b, h, first:] = A.astype(F16)
                B16[b, h] = Bm.astype(F16)
    return Segment(kind, n, codes, scale, zero, mask, svals, A16, B16, ties)


def reconstruct_segment(seg: Segment, g: int) -> np.ndarray:
    """X-hat = D-hat + A B^T + S in fp64 from the stored (fp16) components."""
    if seg.kind == "K":
        Dh = dequant_keys(seg.codes, seg.scale, seg.zero, seg.n if g == 0 else g)
    else:
        Dh = dequant_values(seg.codes, seg.scale, seg.zero, seg.codes.shape[3] if g == 0 else g)
    L = np.einsum("bhnr,bhdr->bhnd", seg.A.astype(F64), seg.Bf.astype(F64))
    return Dh + L + seg.svals.astype(F64)


class OracleCache:
    """The compressed KV cache of one layer: a list of segments per tensor, in
    append order (prefill first, then one segment per flushed buffer)."""

    def __init__(self, B, H_kv, H_q, d_h, bits, group, outlier_ppm, v_per_head=False):
        self.B, self.H_kv, self.H_q, self.d_h = B, H_kv, H_q, d_h
        self.bits, self.group, self.outlier_ppm = bits, group, outlier_ppm      # group 0: per-vector groups
        self.v_per_head = v_per_head
        self.K: List[Segment] = []
        self.V: List[Segment] = []

    @property
    def n_total(self):
        return sum(s.n for s in self.K)

    def compress(self, K16, V16, rank, iters, init_B, v_mask=None, n_lowrank=None):
        """Append one segment.  init_B: fp32 [2,B,H,d,rank] (index 0 = K, 1 = V).
        v_mask: optional precomputed support of S for V (used when this cache holds
        a subset of the heads: Filter ranks a Value token across all heads)."""
        iK = init_B[0] if rank > 0 else None
        iV = init_B[1] if rank > 0 else None
        self.K.append(compress_tensor(K16, "K", self.bits, self.group, self.outlier_ppm, rank, iters, iK,
                                      n_lowrank=n_lowrank))
        self.V.append(compress_tensor(V16, "V", self.bits, self.group, self.outlier_ppm, rank, iters, iV, v_mask,
                                      self.v_per_head, n_lowrank))

    def reconstruct(self):
        """(K-hat, V-hat) fp64 [B,H,n_total,d]."""
        Kh = np.concatenate([reconstruct_segment(s, self.group) for s in self.K], axis=2)
        Vh = np.concatenate([reconstruct_segment(s, self.group) for s in self.V], axis=2)
        return Kh, Vh

    def decompress(self):
        Kh, Vh = self.reconstruct()
        return Kh.astype(F16), Vh.astype(F16)

    def decode_attn(self, q16, K_buf16=None, V_buf16=None, n_buf=0):
        """Eq. 1 for a single query per head: softmax(q K^T / sqrt(d_H)) V over
        every compressed row (rebuilt from its own segment's components) followed
        by the first n_buf rows of the fp16 streaming buffer.  GQA: query head i
        reads KV head floor(i / (H_q/H_kv)).  q16: fp16 [B,H_q,1,d] -> fp16 same."""
        parts_K, parts_V = [], []
        if self.K:
            Kh, Vh = self.reconstruct()
            parts_K.append(Kh)
            parts_V.append(Vh)
        if n_buf > 0:
            parts_K.append(K_buf16[:, :, :n_buf, :].astype(F64))
            parts_V.append(V_buf16[:, :, :n_buf, :].astype(F64))
        Kall = np.concatenate(parts_K, axis=2)
        Vall = np.concatenate(parts_V, axis=2)
        rep = self.H_q // self.H_kv
        out = np.zeros((self.B, self.H_q, 1, self.d_h), F64)
        for b in range(self.B):
            for i in range(self.H_q):
                h = i // rep
                s = (Kall[b, h] @ q16[b, i, 0].astype(F64)) / np.sqrt(F64(self.d_h))
                p = np.exp(s - s.max())
                p /= p.sum()
                out[b, i, 0] = p @ Vall[b, h]
        self.last_attn_f64 = out          # unrounded result, for error reporting
        return out.astype(F16)


def decode_attn_multi(cache: "OracleCache", q16, K_buf16, V_buf16, n_buf, causal=True):
    """Eq. 1 for q_len query rows per head (chunked prefill, speculative decoding): the q_len
    newest tokens are the last q_len of the n_buf buffer rows; every query attends to all
    compressed rows, and query j (0-based) to buffer rows 0 .. n_buf - q_len + j when causal
    (to all n_buf rows otherwise).  q16: fp16 [B,H_q,q_len,d] -> fp64 [B,H_q,q_len,d] (unrounded)."""
    B, Hq, q_len, d = q16.shape
    assert 1 <= q_len <= n_buf or not causal
    Kh, Vh = cache.reconstruct() if cache.K else (np.zeros((B, cache.H_kv, 0, d)), np.zeros((B, cache.H_kv, 0, d)))
    rep = cache.H_q // cache.H_kv
    out = np.zeros((B, Hq, q_len, d), F64)
    for j in range(q_len):
        nb = n_buf - q_len + j + 1 if causal else n_buf
        Kall = np.concatenate([Kh, K_buf16[:, :, :nb, :].astype(F64)], axis=2)
        Vall = np.concatenate([Vh, V_buf16[:, :, :nb, :].astype(F64)], axis=2)
        for b in range(B):
            for i in range(Hq):
                h = i // rep
                s = (Kall[b, h] @ q16[b, i, j].astype(F64)) / np.sqrt(F64(d))
                p = np.exp(s - s.max())
                p /= p.sum()
                out[b, i, j] = p @ Vall[b, h]
    return out


def compressed_bytes(n, d_h, H, bits, g, outlier_ppm, rank, index_bytes=2, v_per_head=False):
    """Byte accounting of one (b, all heads) compressed segment, K + V, against
    its fp16 size (the "KV size" column of Table 1; scale and zero-point in fp16
    as in the KV-cache-component appendix).  g = 0: per-vector groups (one pair
    per Key channel, one per Value token).  index_bytes is this build's own
    choice (the paper's sparse format is "two index vectors and one value
    vector"); it only affects the sparse share."""
    fp16 = 2 * 2 * n * H * d_h
    codes = 2 * n * H * d_h * bits / 8
    if g == 0:
        sz_k = 4 * H * d_h
        sz_v = 4 * n
    else:
        sz_k = 4 * (-(-n // g)) * H * d_h
        sz_v = 4 * n * H * d_h // g
    lowrank = 2 * 2 * (n * rank + d_h * rank) * H
    kv_k, _, _ = outlier_counts(n, outlier_ppm)
    if v_per_head:
        kv_v = H * outlier_counts(d_h, outlier_ppm)[0]
    else:
        kv_v, _, _ = outlier_counts(H * d_h, outlier_ppm)
    sparse = (2 + index_bytes) * (kv_k * H * d_h + kv_v * n)
    total = codes + sz_k + sz_v + lowrank + sparse
    return dict(fp16=fp16, codes=codes, scale_zero=sz_k + sz_v, lowrank=lowrank, sparse=sparse,
                total=total, fraction=total / fp16)
