"""GPU parity on seeded random draws from the space of valid configurations: batch, KV heads, query heads
per KV head, bits, group size (incl. per-vector groups), outlier ratio, ranks, rounds of Algorithm 2,
prefill length (several tiles and a ragged tail, up to the segment lengths where the selection and
power-iteration kernels change path), chunks of 1..n_b tokens, buffer rows, per-head Value Filter.
Same bars as tests/test_gpu_parity.py (its run_case does the comparisons); the draws are fixed by the
seed, so a failure names its case."""
import dataclasses
import random

import pytest

from tests.test_gpu_parity import run_case, say, small_workload

pytestmark = pytest.mark.gpu


def draw(seed):
    r = random.Random(1000 + seed)
    H_kv = r.choice([1, 2, 3, 4, 5, 8])
    gq = r.choice([1, 1, 2, 4, 8])
    B = r.choice([1, 2, 3])
    # lengths around the kernels' path switches (64, 256, 1024) and tile multiples, else anything up to 1600
    n = r.choice([r.randint(1, 70), r.randint(200, 300), r.randint(1000, 1100), r.randint(1, 1600),
                  64 * r.randint(1, 12), 512 * r.randint(1, 3) + r.choice([-1, 0, 1])])
    bits = r.choice([2, 4])
    g = r.choice([0, 32, 64, 128])
    ppm = r.choice([0, 5000, 10000, 20000, 20000, 35000, 80000])
    rank = r.choice([0, 1, 2, 3, 4, 4, 6, 8])
    rank_chunk = r.choice([0, 1, 2, 2, 4])
    n_b = r.choice([4, 20, 20, 33, 64])
    w = dataclasses.replace(small_workload(B=B, H_kv=H_kv, H_q=H_kv * gq, n=n, bits=bits, g=g, ppm=ppm, rank=rank,
                                           seed=7000 + seed, nu=r.choice([3, 4])), rank_chunk=rank_chunk, n_b=n_b)
    kw = dict(n_chunks=r.choice([0, 1, 2, 4]), chunk_n=r.randint(1, n_b), n_buf=r.randint(0, n_b),
              iters=r.choice([1, 2, 3, 3]), v_per_head=r.random() < 0.25)
    return w, kw


@pytest.mark.parametrize("seed", range(48))
def test_random_valid_configuration(seed):
    w, kw = draw(seed)
    say("random case", seed)
    run_case(w, **kw)


@pytest.mark.parametrize("seed", range(8))
def test_random_long_segment(seed):
    """Prefill segments of 2049..9000 tokens (one batch element, one or two KV heads, so that the oracle
    stays fast): the register-resident Key selection with 5..16 chunks and, past 8192 tokens, the
    selection from the channel-major copy; several strips per slab in the Gram pass."""
    r = random.Random(2000 + seed)
    w, kw = draw(100 + seed)
    w = dataclasses.replace(w, B=1, H_kv=r.choice([1, 2]), n=r.choice([r.randint(2049, 9000), 8192 + r.randint(-1, 700)]))
    w = dataclasses.replace(w, H_q=w.H_kv * r.choice([1, 4]))
    say("random long case", seed)
    run_case(w, **kw)


@pytest.mark.parametrize("seed", range(12))
def test_random_multi_query_and_recent_tokens(seed):
    """Random draws for the two entry points that run_case does not reach: the low-rank term on the most recent
    tokens of the prefill call only (gear_compress_recent), then q_len query rows per head (gear_decode_attn_mq)
    over that cache, its chunks and the buffer, with and without the causal rule."""
    import torch

    import gear_workloads as gw
    from tests import parity_util as pu
    from tests.test_gpu_parity import DEV

    r = random.Random(3000 + seed)
    w, kw = draw(200 + seed)
    gq = r.choice([1, 2, 4])
    w = dataclasses.replace(w, H_q=w.H_kv * gq, n=max(w.n, 40), rank=max(w.rank, 1))
    q_len = r.choice([x for x in (1, 2, 4, 8) if x * gq <= 8])
    n_lowrank = r.choice([0, 1, w.n // 4, w.n - 1, w.n])
    n_chunks, chunk_n = kw["n_chunks"], kw["chunk_n"]
    say("random multi-query case", seed, w, "q_len", q_len, "n_lowrank", n_lowrank, kw)
    gc, oc = pu.make_pair(w.B, w.H_kv, w.H_q, w.bits, w.group, w.outlier_ppm, max(w.n_b, chunk_n, q_len), w.n,
                          max(n_chunks, 1), max(w.rank, w.rank_chunk), v_per_head=kw["v_per_head"])
    K, V = gw.make_keys(w, w.n, 0, DEV), gw.make_values(w, w.n, 0, DEV)
    ib = gw.make_init_B(w, w.rank, 0, DEV)
    gc.compress(K, V, w.rank, kw["iters"], ib, n_lowrank=n_lowrank)
    oc.compress(pu.np16(K), pu.np16(V), w.rank, kw["iters"], pu.np16(ib), n_lowrank=n_lowrank)
    for j in range(n_chunks):
        pu.compress_both(gc, oc, gw.make_keys(w, chunk_n, 1 + j, DEV), gw.make_values(w, chunk_n, 1 + j, DEV),
                         w.rank_chunk, kw["iters"], gw.make_init_B(w, w.rank_chunk, 1 + j, DEV))
    rep = pu.compare_components(gc, oc)
    rep.update(pu.compare_decompress(gc, oc))
    if n_lowrank > 0:
        rep.update(pu.compare_lowrank_product(gc, oc, 0))
    cap = gc.cfg.n_buf_cap
    Kb, Vb = gw.make_keys(w, cap, 50, DEV), gw.make_values(w, cap, 50, DEV)
    g = torch.Generator(device="cpu").manual_seed(4000 + seed)
    q = torch.randn(w.B, w.H_q, q_len, 128, generator=g).to(torch.float16).to(DEV)
    for n_buf, causal in ((q_len, True), (r.randint(q_len, cap), True), (r.randint(q_len, cap), False)):
        out = gc.decode_attn_mq(q, Kb, Vb, n_buf, causal)
        want = pu.go.decode_attn_multi(oc, pu.np16(q), pu.np16(Kb), pu.np16(Vb), n_buf, causal)
        rep["mq_%d_%s" % (n_buf, causal)] = pu.check_attention(pu.np16(out), want, "multi-query attention")
    say("  ->", rep)
