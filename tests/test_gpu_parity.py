"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element, on seeded synthetic inputs.  Bars: codes / scale / zero / outlier
support and values bit-exact (off-by-one codes only at counted exact rounding
ties); reconstructed K/V within 1e-3 relative Frobenius of the oracle's;
attention outputs within 2e-3 of the oracle's unrounded fp64 result plus half an fp16 unit in the last place."""
import sys

import numpy as np
import pytest
import torch

import gear_workloads as gw
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def small_workload(B, H_kv, H_q, n, bits, g, ppm, rank, seed, nu=4):
    return gw.Workload("t", B=B, H_kv=H_kv, H_q=H_q, n=n, bits=bits, group=g, outlier_ppm=ppm, rank=rank,
                       rank_chunk=2, n_b=20, steps=1, seed=seed, v_nu=nu)


def run_case(w, n_chunks=1, chunk_n=20, n_buf=7, iters=3, check_attn=True, v_per_head=False):
    say("case", w, "chunks", n_chunks, "chunk_n", chunk_n, "n_buf", n_buf, "v_per_head", v_per_head)
    gc, oc = pu.make_pair(w.B, w.H_kv, w.H_q, w.bits, w.group, w.outlier_ppm, max(w.n_b, chunk_n), w.n,
                          max(n_chunks, 1), max(w.rank, w.rank_chunk), v_per_head=v_per_head)
    K = gw.make_keys(w, w.n, 0, DEV)
    V = gw.make_values(w, w.n, 0, DEV)
    ib = gw.make_init_B(w, w.rank, 0, DEV)
    pu.compress_both(gc, oc, K, V, w.rank, iters, ib)
    rep = pu.compare_components(gc, oc)
    rep.update(pu.compare_decompress(gc, oc))
    if w.rank > 0:
        rep.update(pu.compare_lowrank_product(gc, oc, 0))        # asserts the bound on A B^T
    for j in range(n_chunks):
        Kc = gw.make_keys(w, chunk_n, 1 + j, DEV)
        Vc = gw.make_values(w, chunk_n, 1 + j, DEV)
        ibc = gw.make_init_B(w, w.rank_chunk, 1 + j, DEV)
        pu.compress_both(gc, oc, Kc, Vc, w.rank_chunk, iters, ibc)
    if n_chunks:
        rep.update(pu.compare_components(gc, oc))
        rep.update(pu.compare_decompress(gc, oc))
    if check_attn:
        q = gw.make_queries(w, 0, DEV)
        cap = gc.cfg.n_buf_cap
        Kb = gw.make_keys(w, cap, 50, DEV)
        Vb = gw.make_values(w, cap, 50, DEV)
        rep.update(pu.compare_attention(gc, oc, q, Kb, Vb, n_buf))
        rep["attn_nobuf_vs_f64"] = pu.compare_attention(gc, oc, q)["attn_vs_f64"]
    say("  ->", rep)
    return rep


@pytest.mark.parametrize("bits,g", [(2, 64), (4, 64), (2, 128), (4, 128), (2, 32), (4, 32)])
def test_small_ragged(bits, g):
    w = small_workload(B=2, H_kv=4, H_q=8, n=200, bits=bits, g=g, ppm=20000, rank=4, seed=bits * 10 + g)
    rep = run_case(w, n_chunks=2)
    assert rep["K_nnz"] > 0 and rep["V_nnz"] > 0


@pytest.mark.parametrize("iters", [1, 2, 4])
def test_iteration_counts(iters):
    """L = 1 (the only round is also the last), 2 and 4 rounds of Algorithm 2, on a prefill that
    takes the kernel-per-step path (n > 256) and chunks that take the one-block path."""
    w = small_workload(B=1, H_kv=4, H_q=4, n=300, bits=2, g=64, ppm=20000, rank=4, seed=40 + iters)
    run_case(w, n_chunks=2, iters=iters)


def test_value_lists_in_reserved_and_allocated_regions():
    """s = 2.5 %: the overflow lists of the Value tiles are about as long as their reserved
    regions (48 entries), so some lie there and some are allocated behind them."""
    w = small_workload(B=2, H_kv=8, H_q=8, n=320, bits=2, g=64, ppm=25000, rank=2, seed=77)
    run_case(w, n_chunks=1)


@pytest.mark.parametrize("ppm,rank", [(0, 0), (0, 4), (20000, 0), (10000, 8), (50000, 2), (20000, 3)])
def test_modes(ppm, rank):
    w = small_workload(B=1, H_kv=8, H_q=8, n=300, bits=2, g=64, ppm=ppm, rank=rank, seed=ppm + rank)
    run_case(w, n_chunks=1)


@pytest.mark.parametrize("rank,rank_chunk", [(2, 4), (0, 2), (8, 1), (4, 3)])
def test_chunk_rank_differs_from_prefill_rank(rank, rank_chunk):
    # the decode kernel keeps one copy of the prefill's B factors per block and one per wave for
    # the chunks: both orders of the two ranks, a prefill without factors, and a rank without a
    # vector-read path (3) next to one with it
    import dataclasses
    w = dataclasses.replace(small_workload(B=1, H_kv=4, H_q=8, n=530, bits=2, g=64, ppm=20000, rank=rank,
                                           seed=17 + rank), rank_chunk=rank_chunk)
    run_case(w, n_chunks=5)


@pytest.mark.parametrize("H_kv,H_q,rank,rank_chunk", [(2, 8, 3, 2), (2, 8, 4, 2), (1, 8, 8, 4), (2, 8, 2, 5)])
def test_grouped_queries_with_and_without_one_read_ranks(H_kv, H_q, rank, rank_chunk):
    # four or more query heads per KV head: the decode kernel keeps the low-rank rows in registers
    # when every rank of the launch is 0, 2, 4 or 8 and stages them in LDS otherwise
    import dataclasses
    w = dataclasses.replace(small_workload(B=1, H_kv=H_kv, H_q=H_q, n=300, bits=2, g=64, ppm=20000, rank=rank,
                                           seed=31 + rank), rank_chunk=rank_chunk)
    run_case(w, n_chunks=3)


@pytest.mark.parametrize("n", [1, 7, 20, 63, 64, 65, 513])
def test_token_counts(n):
    w = small_workload(B=1, H_kv=4, H_q=4, n=n, bits=4, g=64, ppm=20000, rank=2, seed=n)
    run_case(w, n_chunks=1, chunk_n=min(20, 13 + n % 5), n_buf=1)


@pytest.mark.parametrize("H_kv,H_q", [(1, 1), (2, 16), (3, 6), (40, 40)])
def test_head_counts(H_kv, H_q):
    w = small_workload(B=1, H_kv=H_kv, H_q=H_q, n=96, bits=2, g=64, ppm=20000, rank=4, seed=H_kv, nu=3)
    run_case(w, n_chunks=1)


@pytest.mark.parametrize("n", [150, 48, 64])
def test_heavy_ties_and_constant_vectors(n):
    """Values on a coarse grid (many exact ties at the Filter threshold and at
    quantizer rounding boundaries), one all-equal head, signed zeros.  n <= 64 takes
    the rank-based selection of short Key vectors, n = 150 the radix selection."""
    w = small_workload(B=1, H_kv=4, H_q=4, n=n, bits=2, g=64, ppm=40000, rank=2, seed=99)
    say("case ties", w)
    gc, oc = pu.make_pair(1, 4, 4, 2, 64, 40000, 20, n, 1, 2)
    g = torch.Generator(device="cpu").manual_seed(5)
    K = (torch.randint(-6, 7, (1, 4, n, 128), generator=g).float() * 0.5)
    V = (torch.randint(-3, 4, (1, 4, n, 128), generator=g).float() * 0.25)
    K[0, 1] = 1.5                                        # constant head
    V[0, 2] = 0.0
    V[0, 2, ::2] = -0.0                                  # signed zeros only
    K = K.to(torch.float16).to(DEV)
    V = V.to(torch.float16).to(DEV)
    ib = gw.make_init_B(w, 2, 0, DEV)
    pu.compress_both(gc, oc, K, V, 2, 3, ib)
    rep = pu.compare_components(gc, oc)
    rep.update(pu.compare_decompress(gc, oc))
    q = gw.make_queries(w, 0, DEV)
    rep.update(pu.compare_attention(gc, oc, q))
    say("  ->", rep)


@pytest.mark.parametrize("n,g,ties", [(1100, 64, False), (2500, 64, True), (4101, 128, False), (8192, 64, True),
                                      (8461, 64, False), (8461, 0, True), (12000, 128, True)])
def test_key_selection_paths_by_segment_length(n, g, ties):
    """The Key Filter (Eq. 4 along the token axis) takes a different kernel by segment length: channel vectors
    in registers (1025 .. 8192 tokens, three sizes) and, beyond, a channel-major copy of the keys read from
    global memory.  Element-wise against the oracle at ragged lengths; `ties`: values on a coarse grid, so
    that the threshold value is shared by many entries and the lowest-index rule decides, with one constant head."""
    bits = 4 if g == 0 else 2
    w = small_workload(B=1, H_kv=2, H_q=2, n=n, bits=bits, g=g, ppm=20000, rank=2, seed=n + g)
    say("case key selection", w, "ties", ties)
    gc, oc = pu.make_pair(1, 2, 2, bits, g, 20000, 20, n, 1, 2)
    if ties:
        gen = torch.Generator(device="cpu").manual_seed(n)
        K = (torch.randint(-6, 7, (1, 2, n, 128), generator=gen).float() * 0.5)
        K[0, 1, :, :7] = 1.5                             # constant channels
        K = K.to(torch.float16).to(DEV)
    else:
        K = gw.make_keys(w, n, 0, DEV)
    V = gw.make_values(w, n, 0, DEV)
    pu.compress_both(gc, oc, K, V, 2, 2, gw.make_init_B(w, 2, 0, DEV))
    rep = pu.compare_components(gc, oc)
    rep.update(pu.compare_decompress(gc, oc))
    rep.update(pu.compare_attention(gc, oc, gw.make_queries(w, 0, DEV)))
    say("  ->", rep)
    assert rep["K_nnz"] > 0


@pytest.mark.parametrize("H_kv,g,ties", [(4, 64, False), (8, 64, True), (2, 0, True), (1, 128, False)])
def test_value_selection_four_token_rows_per_wave(H_kv, g, ties):
    """With at most eight KV heads and at least 16384 tokens in a call the per-token Value Filter (Eq. 4 over the
    token's H_kv * 128 entries) runs four tokens per wave, one per row of 16 lanes.  Element-wise against the oracle
    at a ragged length; `ties`: Values on a coarse grid with constant and signed-zero heads, so that the threshold
    value is shared by many entries (within one side, and between the top and the bottom side)."""
    B = 16 // H_kv * 2
    n = 16384 // B + 37
    bits = 4 if g == 0 else 2
    w = small_workload(B=B, H_kv=H_kv, H_q=H_kv, n=n, bits=bits, g=g, ppm=20000, rank=0, seed=900 + H_kv)
    say("case value rows", w, "ties", ties)
    gc, oc = pu.make_pair(B, H_kv, H_kv, bits, g, 20000, 20, n, 1, 2)
    K = gw.make_keys(w, n, 0, DEV)
    if ties:
        gen = torch.Generator(device="cpu").manual_seed(n)
        V = (torch.randint(-3, 4, (B, H_kv, n, 128), generator=gen).float() * 0.25)
        V[0, 0] = 0.75                                   # constant head
        V[1, H_kv - 1] = 0.0
        V[1, H_kv - 1, ::2] = -0.0                       # signed zeros only
        V = V.to(torch.float16).to(DEV)
    else:
        V = gw.make_values(w, n, 0, DEV)
    pu.compress_both(gc, oc, K, V, 0, 1, None)
    rep = pu.compare_components(gc, oc)
    rep.update(pu.compare_decompress(gc, oc))
    say("  ->", rep)
    assert rep["V_nnz"] > 0


def test_large_magnitudes_inside_the_stated_operand_range():
    """The read feeds q * scale_K and p * scale_V to the matrix cores as fp16 operands (include/gear.h states
    the range: |q * scale_K| < 4094).  Keys of magnitude up to 600, Values up to 1500 and |q| up to 9 give products of up to 3600: the outputs must be finite and agree with the oracle (the softmax is then one-hot)."""
    n = 300
    w = small_workload(B=1, H_kv=2, H_q=4, n=n, bits=2, g=64, ppm=20000, rank=2, seed=77)
    gc, oc = pu.make_pair(1, 2, 4, 2, 64, 20000, 20, n, 1, 2)
    K = (gw.make_keys(w, n, 0, "cpu").float() * 100.0).clamp(-600, 600).to(torch.float16).to(DEV)   # scale_K <= 400
    V = (gw.make_values(w, n, 0, "cpu").float() * 100.0).clamp(-1500, 1500).to(torch.float16).to(DEV)
    pu.compress_both(gc, oc, K, V, 2, 3, gw.make_init_B(w, 2, 0, DEV))
    rep = pu.compare_components(gc, oc)
    q = (gw.make_queries(w, 0, "cpu").float() * 2.0).clamp(-9, 9).to(torch.float16).to(DEV)               # |q * scale_K| <= 3600
    out = gc.decode_attn(q, None, None, 0)
    assert torch.isfinite(out.float()).all()
    rep.update(pu.compare_attention(gc, oc, q))
    say("  ->", rep)


def test_lossless_grid_reconstructs_input_bit_exact():
    gc, oc = pu.make_pair(1, 2, 2, 2, 64, 0, 20, 128, 1, 4)
    g = torch.Generator(device="cpu").manual_seed(6)
    k = torch.randint(0, 4, (1, 2, 128, 128), generator=g)
    k[:, :, 0::64, :] = 0
    k[:, :, 1::64, :] = 3
    K = (-1.0 + 0.5 * k.float()).to(torch.float16).to(DEV)
    v = torch.randint(0, 4, (1, 2, 128, 128), generator=g)
    v[..., 0::64] = 0
    v[..., 1::64] = 3
    V = (2.0 + 0.25 * v.float()).to(torch.float16).to(DEV)
    w = small_workload(1, 2, 2, 128, 2, 64, 0, 4, 7)
    ib = gw.make_init_B(w, 4, 0, DEV)
    pu.compress_both(gc, oc, K, V, 4, 3, ib)
    Kg, Vg = gc.decompress()
    assert torch.equal(Kg, K) and torch.equal(Vg, V)


def test_config0_full():
    w = gw.CONFIGS[0]
    rep = run_case(w, n_chunks=0, n_buf=0, check_attn=False)
    gc, oc = pu.make_pair(w.B, w.H_kv, w.H_q, w.bits, w.group, w.outlier_ppm, w.n_b, w.n, 1, w.rank)
    K = gw.make_keys(w, w.n, 0, DEV)
    V = gw.make_values(w, w.n, 0, DEV)
    ib = gw.make_init_B(w, w.rank, 0, DEV)
    pu.compress_both(gc, oc, K, V, w.rank, w.iters, ib)
    q = gw.make_queries(w, 0, DEV)
    rep = pu.compare_attention(gc, oc, q)          # one decode query, empty buffer
    say("  config0 attention ->", rep)
    # exactly ceil(2% * N) outliers per vector
    mask, _ = gc.export_sparse(0)
    assert (mask.sum(dim=2) == 11).all()           # ceil(0.02*512) per Key channel
    mask, _ = gc.export_sparse(1)
    assert (mask.sum(dim=(1, 3)) == 82).all()      # ceil(0.02*4096) per Value token


def test_repeatable_bitwise():
    """No float atomics on the path: two runs give identical bytes."""
    w = small_workload(B=1, H_kv=4, H_q=8, n=200, bits=2, g=64, ppm=20000, rank=4, seed=3)
    outs = []
    for _ in range(2):
        gc, _ = pu.make_pair(1, 4, 8, 2, 64, 20000, 20, 200, 1, 4)
        K = gw.make_keys(w, 200, 0, DEV)
        V = gw.make_values(w, 200, 0, DEV)
        gc.compress(K, V, 4, 3, gw.make_init_B(w, 4, 0, DEV))
        Kh, Vh = gc.decompress()
        o = gc.decode_attn(gw.make_queries(w, 0, DEV))
        outs.append((Kh.clone(), Vh.clone(), o.clone()))
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)


def test_rank_deficient_residual():
    """A residual of exact rank 1 under a rank-4 solver: codes on a lossless grid plus u v^T small
    enough to leave every code, scale and zero-point alone, so R = u v^T exactly.  Both sides must
    drop the three dependent directions (QR of B, then of A) and return A B^T = R."""
    n = 300
    w = small_workload(1, 2, 2, n, 2, 64, 0, 4, 71)
    gc, oc = pu.make_pair(1, 2, 2, 2, 64, 0, 20, n, 1, 4)
    g = torch.Generator(device="cpu").manual_seed(8)
    step = 2.0 ** -10
    k = torch.randint(1, 3, (1, 2, n, 128), generator=g)     # inner codes only, so the perturbed values stay inside the range
    k[:, :, 0::64, :] = 0                                    # every Key group holds its end points ...
    k[:, :, 1::64, :] = 3
    u = torch.randint(-7, 8, (1, 2, n, 1), generator=g).float()   # (3 x, 5 x, 7 x: products that round in fp32)
    u[:, :, 0::64] = 0                                       # ... in rows the perturbation leaves alone
    u[:, :, 1::64] = 0
    vk = torch.randint(1, 3, (1, 2, 1, 128), generator=g).float() * step
    K = (-1.0 + 0.5 * k.float() + u * vk).to(torch.float16)
    v = torch.randint(1, 3, (1, 2, n, 128), generator=g)
    v[..., 0::64] = 0                                        # Value groups run along the channels
    v[..., 1::64] = 3
    uv = torch.randint(-7, 8, (1, 2, n, 1), generator=g).float()
    vv = torch.randint(1, 3, (1, 2, 1, 128), generator=g).float() * step
    vv[..., 0::64] = 0
    vv[..., 1::64] = 0
    V = (-1.0 + 0.5 * v.float() + uv * vv).to(torch.float16)
    assert torch.equal(K.float(), -1.0 + 0.5 * k.float() + u * vk)      # the construction is exact in fp16
    ib = gw.make_init_B(w, 4, 0, DEV)
    pu.compress_both(gc, oc, K.to(DEV), V.to(DEV), 4, 3, ib)
    rep = pu.compare_components(gc, oc)
    # the oracle's factors reproduce the rank-1 residual, with three zero columns
    Lo = np.einsum("bhnr,bhdr->bhnd", oc.K[0].A.astype(np.float64), oc.K[0].Bf.astype(np.float64))
    assert np.abs(Lo - (u * vk).numpy()).max() <= 2e-3 * step * 14
    assert (np.abs(oc.K[0].A.astype(np.float64)).sum(axis=2) > 0).sum(axis=-1).max() == 1
    rep.update(pu.compare_lowrank_product(gc, oc, 0))
    rep.update(pu.compare_decompress(gc, oc))
    A, Bf = gc.export_lowrank(0, 0)
    assert torch.isfinite(A.float()).all() and torch.isfinite(Bf.float()).all()
    rep.update(pu.compare_attention(gc, oc, gw.make_queries(w, 0, DEV)))
    say("  ->", rep)


def test_seeded_start_matrix():
    """init_B = NULL: the library draws the start matrices of Algorithm 2 from the seed.  The stored
    factors must equal, bit for bit, those of a call that is handed the same numbers as an array
    (the generator's integer formula, mirrored in gear_workloads), and match the oracle run on it."""
    w = small_workload(B=2, H_kv=3, H_q=3, n=400, bits=2, g=64, ppm=20000, rank=4, seed=91)
    K = gw.make_keys(w, w.n, 0, DEV)
    V = gw.make_values(w, w.n, 0, DEV)
    Kc = gw.make_keys(w, 20, 1, DEV)
    Vc = gw.make_values(w, 20, 1, DEV)
    seed, seed_c = 0x1234567890ABCDEF, 7
    ib = gw.make_init_B_hashed(seed, w.B, w.H_kv, 4, DEV)
    ibc = gw.make_init_B_hashed(seed_c, w.B, w.H_kv, 3, DEV)
    assert float(ib.min()) >= -1.0 and float(ib.max()) < 1.0 and abs(float(ib.mean())) < 0.02
    gc, oc = pu.make_pair(w.B, w.H_kv, w.H_q, 2, 64, 20000, 20, w.n, 1, 4)
    pu.compress_both(gc, oc, K, V, 4, 3, ib)
    pu.compress_both(gc, oc, Kc, Vc, 3, 3, ibc)
    gs, _ = pu.make_pair(w.B, w.H_kv, w.H_q, 2, 64, 20000, 20, w.n, 1, 4)
    gs.compress(K, V, 4, 3, None, seed=seed)               # prefill: the kernel-per-step path
    gs.compress(Kc, Vc, 3, 3, None, seed=seed_c)           # chunk: the one-block path
    for which in (0, 1):
        for seg in (0, 1):
            A1, B1 = gc.export_lowrank(which, seg)
            A2, B2 = gs.export_lowrank(which, seg)
            assert torch.equal(A1, A2) and torch.equal(B1, B2), (which, seg)
    rep = pu.compare_lowrank_product(gc, oc, 0)
    rep.update(pu.compare_decompress(gc, oc))
    say("  ->", rep)


# ---- the per-head Value Filter and the per-vector grouping ("KCVT") ----
@pytest.mark.parametrize("bits,ppm,rank", [(4, 20000, 4), (2, 20000, 2), (4, 0, 4), (4, 20000, 0), (2, 50000, 8)])
def test_per_vector_groups(bits, ppm, rank):
    """group = 0: one group per Key channel over the tokens of a call, one per Value token over all heads
    (the paper's 4-bit backbone).  n = 300 takes the kernel-per-step power iteration, the chunks the one-block one."""
    w = small_workload(B=2, H_kv=4, H_q=8, n=300, bits=bits, g=0, ppm=ppm, rank=rank, seed=300 + bits + rank)
    rep = run_case(w, n_chunks=2)
    assert ppm == 0 or (rep["K_nnz"] > 0 and rep["V_nnz"] > 0)


@pytest.mark.parametrize("bits,g,ppm,rank", [(2, 64, 20000, 4), (4, 128, 20000, 2), (2, 32, 100000, 4), (4, 0, 20000, 4),
                                             (2, 0, 300000, 2)])
def test_value_filter_per_head(bits, g, ppm, rank):
    """Filter_s ranks every head's 128 channels of a Value token on their own: exactly ceil(s * 128) outliers
    per (head, token); with g = 0 together with the per-vector grouping."""
    w = small_workload(B=2, H_kv=3, H_q=6, n=280, bits=bits, g=g, ppm=ppm, rank=rank, seed=400 + bits + rank)
    run_case(w, n_chunks=1, v_per_head=True)
    gc, _ = pu.make_pair(2, 3, 6, bits, g, ppm, 20, 280, 1, rank, v_per_head=True)
    gc.compress(gw.make_keys(w, 280, 0, DEV), gw.make_values(w, 280, 0, DEV), rank, 3, gw.make_init_B(w, rank, 0, DEV))
    mask, _ = gc.export_sparse(1)
    assert (mask.sum(dim=3) == -(-ppm * 128 // 1000000)).all()


def test_per_vector_groups_ties_and_constants():
    """Coarse value grid, one constant head, signed zeros, under the per-vector grouping and the per-head Filter."""
    n = 150
    w = small_workload(B=1, H_kv=4, H_q=4, n=n, bits=4, g=0, ppm=40000, rank=2, seed=98)
    gc, oc = pu.make_pair(1, 4, 4, 4, 0, 40000, 20, n, 1, 2, v_per_head=True)
    g = torch.Generator(device="cpu").manual_seed(15)
    K = (torch.randint(-6, 7, (1, 4, n, 128), generator=g).float() * 0.5)
    V = (torch.randint(-3, 4, (1, 4, n, 128), generator=g).float() * 0.25)
    K[0, 1] = 1.5
    V[0, 2] = 0.0
    V[0, 2, ::2] = -0.0
    K = K.to(torch.float16).to(DEV)
    V = V.to(torch.float16).to(DEV)
    pu.compress_both(gc, oc, K, V, 2, 3, gw.make_init_B(w, 2, 0, DEV))
    rep = pu.compare_components(gc, oc)
    rep.update(pu.compare_decompress(gc, oc))
    rep.update(pu.compare_attention(gc, oc, gw.make_queries(w, 0, DEV)))
    say("  ->", rep)


# ---- multi-query read (q_len query rows per head) ----
@pytest.mark.parametrize("H_kv,H_q,q_len,causal", [(2, 2, 4, True), (2, 2, 8, True), (2, 4, 2, True), (2, 4, 4, False),
                                                   (1, 4, 2, True), (3, 3, 1, True)])
def test_multi_query_read(H_kv, H_q, q_len, causal):
    """q_len query rows per head against the oracle's per-row attention: every row sees the whole compressed
    cache (prefill + chunks) and, when causal, the buffer rows up to its own token."""
    w = small_workload(B=2, H_kv=H_kv, H_q=H_q, n=700, bits=2, g=64, ppm=20000, rank=4, seed=500 + q_len + H_q)
    gc, oc = pu.make_pair(w.B, H_kv, H_q, 2, 64, 20000, 20, w.n, 2, 4)
    pu.compress_both(gc, oc, gw.make_keys(w, w.n, 0, DEV), gw.make_values(w, w.n, 0, DEV), 4, 3, gw.make_init_B(w, 4, 0, DEV))
    for j in range(2):
        pu.compress_both(gc, oc, gw.make_keys(w, 20, 1 + j, DEV), gw.make_values(w, 20, 1 + j, DEV), 2, 3,
                         gw.make_init_B(w, 2, 1 + j, DEV))
    Kb, Vb = gw.make_keys(w, 20, 50, DEV), gw.make_values(w, 20, 50, DEV)
    g = torch.Generator(device="cpu").manual_seed(600 + q_len)
    q = torch.randn(w.B, H_q, q_len, 128, generator=g).to(torch.float16).to(DEV)
    for n_buf in (q_len, 13 if q_len <= 13 else 20, 20):
        out = gc.decode_attn_mq(q, Kb, Vb, n_buf, causal)
        want = pu.go.decode_attn_multi(oc, pu.np16(q), pu.np16(Kb), pu.np16(Vb), n_buf, causal)
        rep = pu.check_attention(pu.np16(out), want, "multi-query attention")
        say("  q_len", q_len, "heads", H_kv, H_q, "causal", causal, "n_buf", n_buf, "->", rep)
    if q_len == 1:      # one row: the same launch as the single-query entry point
        assert torch.equal(gc.decode_attn_mq(q, Kb, Vb, 7, True), gc.decode_attn(q, Kb, Vb, 7))


def test_multi_query_read_argument_checks():
    cfg = pu.gb.make_config(1, 2, 8, 2, 64, 0, 20, 64, 1, 0)
    gc = pu.gb.GearCache(cfg, DEV)
    gc.compress(torch.zeros(1, 2, 64, 128, dtype=torch.float16, device=DEV), torch.zeros(1, 2, 64, 128, dtype=torch.float16, device=DEV), 0, 3)
    Kb = torch.zeros(1, 2, 20, 128, dtype=torch.float16, device=DEV)
    for q_len, n_buf in ((3, 20), (4, 20), (2, 1)):      # not a power of two; 4 heads x 4 rows > 8 columns; fewer buffer rows than queries
        q = torch.zeros(1, 8, q_len, 128, dtype=torch.float16, device=DEV)
        with pytest.raises(pu.gb.GearError) as e:
            gc.decode_attn_mq(q, Kb, Kb, n_buf, True)
        assert e.value.status == pu.gb.GEAR_EINVAL


# ---- error reduction on part of the tokens (the ablations of Sec. 4.3) ----
@pytest.mark.parametrize("n,n_lowrank", [(600, 150), (600, 1), (600, 0), (600, 600), (200, 77)])
def test_low_rank_on_recent_tokens_only(n, n_lowrank):
    """gear_compress_recent: SVDSolver on the residual rows of the n_lowrank most recent tokens; earlier tokens get
    A = 0.  n = 600 takes the Gram-matrix path, n = 200 the one-block path."""
    w = small_workload(B=2, H_kv=2, H_q=4, n=n, bits=2, g=64, ppm=20000, rank=4, seed=700 + n_lowrank)
    gc, oc = pu.make_pair(2, 2, 4, 2, 64, 20000, 20, n, 1, 4)
    K, V = gw.make_keys(w, n, 0, DEV), gw.make_values(w, n, 0, DEV)
    ib = gw.make_init_B(w, 4, 0, DEV)
    gc.compress(K, V, 4, 3, ib, n_lowrank=n_lowrank)
    oc.compress(pu.np16(K), pu.np16(V), 4, 3, pu.np16(ib), n_lowrank=n_lowrank)
    rep = pu.compare_components(gc, oc)
    rep.update(pu.compare_decompress(gc, oc))
    if n_lowrank > 0:
        rep.update(pu.compare_lowrank_product(gc, oc, 0))
        A, _ = gc.export_lowrank(0, 0)
        assert not A[:, :, :n - n_lowrank].any()
    else:
        assert gc.cache.rank_prefill == 0
    rep.update(pu.compare_attention(gc, oc, gw.make_queries(w, 0, DEV)))
    say("  ->", rep)


def test_error_reduction_on_prefill_tokens_only():
    """"GEAR-L Prefill": the flushed buffers are stored with rank 0 and without outliers' help from a low-rank term;
    the decode kernel then mixes a rank-4 prefill segment with rank-0 chunks."""
    import dataclasses
    w = dataclasses.replace(small_workload(B=1, H_kv=4, H_q=8, n=530, bits=2, g=64, ppm=0, rank=4, seed=88), rank_chunk=0)
    run_case(w, n_chunks=5)
