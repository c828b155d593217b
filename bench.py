#!/usr/bin/env python3
"""Benchmark of the GEAR hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic KV of the
headline workload (by default config 4, the Llama-3-8B GQA layer shape: the largest
configuration that one GPU holds):
  1. gear_compress of the n-token prefill (Filter, Quant, power iteration),
  2. n_b decode iterations: the new token's k/v row is already in its buffer
     slot (the push is the caller writing that row), then gear_decode_attn over
     the compressed cache + the buffer rows so far,
  3. gear_compress of the full buffer as a new chunk (rank r_g).
Decode iterations read cache replicas that hold the prefill segment plus
--chunks appended chunks (default: half of the flushes of the config's decode
run, i.e. the cache as it is in the middle of that run) and rotate over three
replicas, so their reads come from HBM and not from the 256 MB Infinity Cache.

After the timed steps of the headline workload every other configuration gets a
short run of the same measurement (`per_config`), and the CPU oracle is timed on a
sample of the headline workload (`cpu_baseline`).

Prints ONE JSON line.  value = KV compress GB/s (fp16 K+V input bytes of the
prefill / time of its gear_compress call); the decode-attention rate is given
beside it.  Both carry their fraction of the 8 TB/s HBM roofline computed from
ALGORITHMIC bytes (one read of the input plus the compressed output for
compress; the compressed cache plus live buffer rows for decode).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def outlier_count(n_v, ppm):
    return min(n_v, -((-ppm * n_v) // 1_000_000))


def compressed_bytes(w, n, rank):
    """Algorithmic bytes of one compressed segment of n tokens, K + V, whole batch."""
    slabs = w.B * w.H_kv
    d = w.d_h
    codes = 2 * slabs * n * d * w.bits // 8
    if w.group == 0:      # per-vector groups: one pair per Key channel, one per Value token over all heads
        sz = 4 * slabs * d + 4 * w.B * n
    else:
        sz = slabs * (4 * (-(-n // w.group)) * d + 4 * n * d // w.group)
    lowrank = 2 * slabs * (2 * n * rank + 2 * d * rank)
    v_out = w.H_kv * outlier_count(d, w.outlier_ppm) if w.v_per_head else outlier_count(w.H_kv * d, w.outlier_ppm)
    sparse = 4 * (slabs * d * outlier_count(n, w.outlier_ppm) + w.B * n * v_out)
    return codes + sz + lowrank + sparse


# SURVEY-table bars: bytes the method itself must move -> time at 60 % (compress) / 70 % (decode) of 8 TB/s
def bar_times(w, in_bytes, comp_bytes, dec_bytes):
    return {"compress_us_at_60pct": round((in_bytes + comp_bytes) / (0.6 * HBM_PEAK_GBPS * 1e9) * 1e6, 1),
            "decode_us_at_70pct": round(dec_bytes / (0.7 * HBM_PEAK_GBPS * 1e9) * 1e6, 1)}


def measure(w, steps, warmup, chunks, dev):
    """Runs `warmup` untimed and `steps` timed passes of the whole hot path on workload w.
    Returns the per-call averages (HIP events on the caller's stream) and the wall time."""
    import torch
    import gear_workloads as gw
    from paper_2403_05527_amd import binding as gb
    NREP = 3
    pre_chunks = chunks if chunks >= 0 else (w.steps // w.n_b) // 2
    max_chunks = max(pre_chunks, 1)
    cfg = gb.make_config(w.B, w.H_kv, w.H_q, w.bits, w.group, w.outlier_ppm, w.n_b, w.n, max_chunks,
                         max(w.rank, w.rank_chunk), flags=gb.GEAR_FLAG_V_FILTER_PER_HEAD if w.v_per_head else 0)
    K = gw.make_keys(w, w.n, 0, dev)
    V = gw.make_values(w, w.n, 0, dev)
    ib = gw.make_init_B(w, w.rank, 0, dev)
    ibc = gw.make_init_B(w, w.rank_chunk, 1, dev)
    Kb = gw.make_keys(w, w.n_b, 1, dev)          # decode-time tokens, one buffer's worth
    Vb = gw.make_values(w, w.n_b, 1, dev)
    qs = [gw.make_queries(w, i, dev) for i in range(w.n_b)]
    out = torch.empty_like(qs[0])
    pre = gb.GearCache(cfg, dev)                 # target of the timed prefill compress
    reps = [gb.GearCache(cfg, dev) for _ in range(NREP)]   # caches the decode iterations read
    n_lr = -(-w.n * w.lowrank_recent_pct // 100)       # prefill tokens that take the low-rank term (all of them by default)
    n_lr = None if n_lr >= w.n else n_lr
    for r in reps:
        r.compress(K, V, w.rank, w.iters, ib, n_lowrank=n_lr)
        for _ in range(pre_chunks):
            r.compress(Kb, Vb, w.rank_chunk, w.iters, ibc if w.rank_chunk > 0 else None)
    torch.cuda.synchronize()

    in_bytes = 2 * K.numel() * 2
    comp_bytes = compressed_bytes(w, w.n, w.rank)
    chunk_bytes = compressed_bytes(w, w.n_b, w.rank_chunk)
    row_bytes = 2 * w.B * w.H_kv * w.d_h * 2          # one k row + one v row per slab
    qo_bytes = 2 * w.B * w.H_q * w.d_h * 2
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(i, record):
        e0, e1 = ev(), ev()
        pre.reset()
        e0.record()
        pre.compress(K, V, w.rank, w.iters, ib, n_lowrank=n_lr)
        e1.record()
        devs = []
        for t in range(w.n_b):
            d = reps[(i * w.n_b + t) % NREP]     # rotate: each read of a replica follows reads of the other two
            a, b = ev(), ev()
            a.record()
            d.decode_attn(qs[t], Kb, Vb, t + 1, out)
            b.record()
            devs.append((a, b, d.cache.n_chunks, t + 1))
        c0, c1 = ev(), ev()
        c0.record()
        pre.compress(Kb, Vb, w.rank_chunk, w.iters, ibc if w.rank_chunk > 0 else None)     # the flush: the buffer becomes a chunk of the fresh cache
        c1.record()
        return (e0, e1, devs, c0, c1) if record else None

    for i in range(warmup):
        step(i, False)
    torch.cuda.synchronize()
    recs = []
    t0 = time.perf_counter()
    for i in range(steps):
        recs.append(step(warmup + i, True))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_comp, t_dec, t_chunk, dec_bytes = [], [], [], []
    for (e0, e1, devs, c0, c1) in recs:
        t_comp.append(e0.elapsed_time(e1) * 1e-3)
        t_chunk.append(c0.elapsed_time(c1) * 1e-3)
        for (a, b, n_chunks, n_buf) in devs:
            t_dec.append(a.elapsed_time(b) * 1e-3)
            dec_bytes.append(comp_bytes + n_chunks * chunk_bytes + n_buf * row_bytes + qo_bytes)
    mean = lambda x: sum(x) / len(x)
    # the multi-query read (q_len rows per head in one pass over the cache), with as many rows as fit the
    # kernel's eight query columns per KV head; same replicas, same rotation
    mq = None
    q_len = 8 // (w.H_q // w.H_kv)
    if q_len > 1:
        qm = torch.randn(w.B, w.H_q, q_len, w.d_h, device=dev).to(torch.float16)
        om = torch.empty_like(qm)
        for i in range(3):
            reps[i % NREP].decode_attn_mq(qm, Kb, Vb, w.n_b, True, om)
        a, b = ev(), ev()
        a.record()
        for i in range(12):
            reps[i % NREP].decode_attn_mq(qm, Kb, Vb, w.n_b, True, om)
        b.record()
        torch.cuda.synchronize()
        tm = a.elapsed_time(b) * 1e-3 / 12
        mq = {"q_len": q_len, "us": round(tm * 1e6, 2), "query_rows_per_s": round(w.B * q_len / tm, 1)}
    arena_bytes = pre.arena_bytes
    res = {"w": w, "wall": wall, "tc": mean(t_comp), "td": mean(t_dec), "tchunk": mean(t_chunk),
           "dec_bytes": mean(dec_bytes), "in_bytes": in_bytes, "comp_bytes": comp_bytes, "pre_chunks": pre_chunks,
           "arena_bytes": arena_bytes, "mq": mq, "sample": (K[:16].cpu(), V[:16].cpu(), ib[:, :16].cpu(), qs[0][:16].cpu())}
    del pre, reps, K, V, Kb, Vb, qs
    torch.cuda.empty_cache()
    return res


def summarize(m):
    w = m["w"]
    comp_algo_gbps = (m["in_bytes"] + m["comp_bytes"]) / m["tc"] / 1e9
    dec_algo_gbps = m["dec_bytes"] / m["td"] / 1e9
    d = {"workload": w.name, "compress_ms": round(m["tc"] * 1e3, 4), "compress_input_gbps": round(m["in_bytes"] / m["tc"] / 1e9, 1),
         "compress_frac": round(comp_algo_gbps / HBM_PEAK_GBPS, 4),
         "chunk_compress_ms": round(m["tchunk"] * 1e3, 4),
         "decode_attn_us": round(m["td"] * 1e6, 2), "decode_attn_tokens_per_s": round(w.B / m["td"], 1),
         "decode_frac": round(dec_algo_gbps / HBM_PEAK_GBPS, 4),
         "decode_loop_tokens_per_s": round(w.B * w.n_b / (w.n_b * m["td"] + m["tchunk"]), 1),
         "compressed_fraction_algorithmic": round(m["comp_bytes"] / m["in_bytes"], 4),
         "arena_fraction": round(m["arena_bytes"] / m["in_bytes"], 4)}
    d.update(bar_times(w, m["in_bytes"], m["comp_bytes"], m["dec_bytes"]))
    if m.get("mq"):
        d["decode_multi_query"] = m["mq"]
    return d


def read_traffic(name):
    """HBM bytes per decode launch from rocprofv3 counters (FETCH_SIZE + WRITE_SIZE, scaled by a streaming kernel of
    known size), measured offline per workload; the file gives the commands."""
    tf = os.path.join(ROOT, "profiles", "decode_split_%s_hbm_traffic.txt" % name)
    if os.path.exists(tf):
        for line in open(tf):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1])
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4, help="index into gear_workloads.CONFIGS of the headline workload "
                    "(default: config 4, the largest one-GPU configuration)")
    ap.add_argument("--chunks", type=int, default=-1, help="appended chunks in the caches the decode steps read")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the short runs of the other configurations")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="kept for the profiling commands: the plain streaming kernel over 1 GiB (reads 1 GiB and "
                         "writes 1 GiB: out = in + 1 on bytes) that the rocprofv3 FETCH_SIZE / WRITE_SIZE readings "
                         "are scaled by runs after every timed region")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path would shard over the batch with no "
              "exchange between GPUs); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import gear_workloads as gw
    from paper_2403_05527_amd import binding as gb

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    gb.load_library()
    dev = "cuda:0"
    w = gw.CONFIGS[args.config]
    m = measure(w, args.steps, args.warmup, args.chunks, dev)
    head = summarize(m)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    dec_algo_gbps = m["dec_bytes"] / m["td"] / 1e9
    comp_algo_gbps = (m["in_bytes"] + m["comp_bytes"]) / m["tc"] / 1e9
    res = {
        "metric": "KV compress GB/s + compressed-KV decode attn tokens/s; % of HBM roofline",
        "value": round(m["in_bytes"] / m["tc"] / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(m["wall"] / args.steps * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H_kv": w.H_kv, "H_q": w.H_q, "d_h": w.d_h, "n": w.n,
                   "bits": w.bits, "group": w.group, "outlier_ppm": w.outlier_ppm, "rank": w.rank,
                   "rank_chunk": w.rank_chunk, "n_b": w.n_b, "iters": w.iters,
                   "chunks_in_decoded_cache": m["pre_chunks"]},
        "compress_ms": head["compress_ms"],
        "chunk_compress_ms": head["chunk_compress_ms"],
        "decode_attn_us": head["decode_attn_us"],
        "decode_attn_tokens_per_s": head["decode_attn_tokens_per_s"],
        # the streaming loop: n_b decode steps and the flush of the full buffer into a chunk
        "decode_loop_tokens_per_s": head["decode_loop_tokens_per_s"],
        "compressed_fraction_algorithmic": head["compressed_fraction_algorithmic"],
        "arena_fraction": head["arena_fraction"],
        "roofline": {"bound": "hbm", "kernel": "gear_decode_attn (decode_split_kernel + combine)",
                     "achieved": round(dec_algo_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(dec_algo_gbps / HBM_PEAK_GBPS, 4), "traffic": read_traffic(w.name) if args.chunks < 0 else None,
                     "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE)",
                     "algorithmic_bytes_per_launch": int(m["dec_bytes"])},
        "roofline_compress": {"bound": "hbm", "kernel": "gear_compress (all kernels of the call)",
                              "achieved": round(comp_algo_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                              "frac": round(comp_algo_gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                              "algorithmic_bytes_per_call": int(m["in_bytes"] + m["comp_bytes"])},
    }
    # a plain streaming kernel on the same box (out = in + 1 over 1 GiB of bytes: 1 GiB read + 1 GiB written),
    # the practical ceiling next to the nominal peak; --calibrate-copy also uses it to scale the profiler's counters
    src = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.add(src, 1, out=dst)
    s0, s1 = ev(), ev()
    s0.record()
    for _ in range(5):
        torch.add(src, 1, out=dst)
    s1.record()
    torch.cuda.synchronize()
    res["roofline"]["measured_stream_gbps"] = round(5 * 2 * (1 << 30) / (s0.elapsed_time(s1) * 1e-3) / 1e9, 1)
    del src, dst
    torch.cuda.empty_cache()
    sample = m.pop("sample")
    if not args.no_per_config:
        # the other configurations: a short run each (1 warm-up + 3 passes), same measurement
        per = []
        for i, wi in enumerate(gw.CONFIGS):
            if i == 0:
                continue                              # config 0 is the small parity case (launch-latency bound)
            if i == args.config:
                per.append(head)
                continue
            mi = measure(wi, 3, 1, -1, dev)
            mi.pop("sample")
            per.append(summarize(mi))
        for wi in gw.VARIANTS:                        # per-vector groups / per-head Value Filter
            mi = measure(wi, 3, 1, -1, dev)
            mi.pop("sample")
            per.append(summarize(mi))
        res["per_config"] = per
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, *sample)
    print(json.dumps(res), flush=True)


def _oracle_pass(args):
    """One batch element through the oracle: one compress, then `reads` decode reads.  Returns the two times."""
    w, Kh, Vh, ibh, qh, reads = args
    from threadpoolctl import threadpool_limits
    from oracle import gear_oracle as go
    with threadpool_limits(limits=1):
        oc = go.OracleCache(1, w.H_kv, w.H_q, w.d_h, w.bits, w.group, w.outlier_ppm, w.v_per_head)
        t0 = time.perf_counter()
        oc.compress(Kh, Vh, w.rank, w.iters, ibh)
        tc = time.perf_counter() - t0
        t0 = time.perf_counter()
        for _ in range(reads):
            oc.decode_attn(qh)
        td = (time.perf_counter() - t0) / max(reads, 1)
    return tc, td


def cpu_baseline(w, K, V, ib, q):
    """The oracle as it stands, timed on the host cores on a sample of whole batch elements of the same
    workload (all heads; the Value Filter couples them): one element on one thread, then one element per
    core on all cores at once (numpy releases the interpreter lock inside its array operations; every
    worker is held to one thread of the numeric libraries)."""
    from concurrent.futures import ThreadPoolExecutor
    cores = len(os.sched_getaffinity(0))
    nb = min(cores, K.shape[0])
    items = [(w, K[b:b + 1].numpy(), V[b:b + 1].numpy(), ib[:, b:b + 1].numpy(), q[b:b + 1].numpy(), 2) for b in range(nb)]
    tc1, td1 = _oracle_pass(items[0])
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=nb) as ex:
        times = list(ex.map(_oracle_pass, items))
    wall = time.perf_counter() - t0
    el_bytes = 2 * K[:1].numel() * 2
    tc_all = sum(t[0] for t in times) / nb            # mean time of a compress while all workers run
    td_all = sum(t[1] for t in times) / nb
    return {"value": round(nb * el_bytes / tc_all / 1e9, 5), "unit": "GB/s", "cores": nb, "kind": "oracle",
            "host_cores_available": cores,
            "decode_attn_tokens_per_s": round(nb / td_all, 3),
            "single_thread": {"value": round(el_bytes / tc1 / 1e9, 5), "unit": "GB/s", "cores": 1,
                              "decode_attn_tokens_per_s": round(1.0 / td1, 3)},
            "sample": "%d of %d batch elements (all %d KV heads, n=%d), one per worker thread, each one compress + 2 decode "
                      "reads, numpy oracle with its numeric libraries held to 1 thread per worker: %.1f s wall; before "
                      "that one element alone on one thread: compress %.1f s, decode read %.2f s"
                      % (nb, w.B, w.H_kv, w.n, wall, tc1, td1)}


if __name__ == "__main__":
    main()
