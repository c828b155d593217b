"""The library's kernels and launchers, compiled as plain C++ against the CPU stand-in
for the HIP device environment in tests/simt/ and run under the address sanitizer:
one small end-to-end case (prefill compress, one chunk, decode attention over cache +
buffer, decompress) through the C ABI, compared with the oracle.  This checks the host
logic (grids, LDS sizes, arena and workspace layout) and that no kernel reads or
writes outside its buffers or its LDS; it does not replace the GPU parity tests (the
emulation knows nothing of the real compiler's code or the hardware's timing)."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import gear_workloads as gw
from oracle import gear_oracle as go
from tests import parity_util as pu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SIMT = os.path.join(ROOT, "tests", "simt")
CSRC = os.path.join(ROOT, "paper_2403_05527_amd", "csrc")
SOURCES = ["gear_api", "compress_filter", "compress_values", "lowrank", "decode", "decompress_export"]


def find_clang():
    for c in ("/opt/rocm/llvm/bin/clang++", shutil.which("clang++")):
        if c and os.path.exists(c):
            return c
    return None


@pytest.fixture(scope="module")
def emulator(tmp_path_factory):
    cxx = find_clang()
    if cxx is None:
        pytest.skip("no clang++ to build the CPU emulation")
    out = tmp_path_factory.mktemp("simt")
    # -ffp-contract=fast: the host compiler may fuse every multiply-add it finds, except where the sources
    # switch contraction off (the quantizer's decision sequence), which the bit-exact code comparison checks
    flags = ["-std=c++17", "-O1", "-g", "-ffp-contract=fast", "-fsanitize=address", "-fno-omit-frame-pointer", "-pthread",
             "-I", SIMT, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    procs = []
    objs = []
    for s in SOURCES:
        o = str(out / (s + ".o"))
        objs.append(o)
        procs.append(subprocess.Popen([cxx, "-x", "c++", "-c", os.path.join(CSRC, s + ".hip"), "-o", o] + flags,
                                      stderr=subprocess.PIPE, text=True))
    for s in ("simt_rt", "run_pipeline"):
        o = str(out / (s + ".o"))
        objs.append(o)
        procs.append(subprocess.Popen([cxx, "-c", os.path.join(SIMT, s + ".cpp"), "-o", o] + flags,
                                      stderr=subprocess.PIPE, text=True))
    for p in procs:
        err = p.communicate()[1]
        assert p.returncode == 0, err[-3000:]
    exe = str(out / "run_pipeline")
    r = subprocess.run([cxx] + objs + ["-o", exe] + flags, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    return exe


@pytest.mark.parametrize("B,H,Hq,n,bits,g,ppm,rank,n_buf,per_head,chunk_n,n_b,n_lowrank", [
    (1, 4, 8, 290, 2, 64, 20000, 4, 5, False, 20, 20, -1),     # the method as stated; n > 256: Gram-matrix power iteration
    (1, 2, 2, 140, 4, 0, 30000, 2, 3, True, 20, 20, -1),       # per-vector groups and the per-head Value Filter
    (1, 8, 8, 70, 2, 64, 20000, 2, 3, False, 20, 20, -1),      # eight KV heads: Value token rows of 1024 entries, four per wave
    (1, 2, 2, 200, 4, 32, 30000, 2, 3, False, 20, 20, -1),     # two KV heads by the same kernel, 4-bit codes, groups of 32
    (1, 1, 2, 70, 2, 64, 20000, 2, 255, False, 255, 255, -1),  # the largest streaming buffer: 255 live rows, a flushed
                                                           # segment of 255 tokens (two 128-row pieces in the decode kernel)
    (1, 2, 8, 1100, 2, 128, 10000, 8, 7, False, 20, 20, -1),   # n > 1024: Key vectors selected in registers; rank 8, four
                                                           # query heads per KV head, groups of 128
    (1, 1, 8, 150, 4, 64, 20000, 3, 4, False, 33, 40, -1),     # eight query heads per KV head, a rank that is not one read
                                                           # (factor rows staged in LDS), a flushed segment of 33 tokens
    (1, 2, 4, 330, 2, 64, 20000, 4, 6, False, 20, 20, 100),  # the low-rank term on the last 100 of 330 tokens only
])
def test_pipeline_under_address_sanitizer(emulator, tmp_path, B, H, Hq, n, bits, g, ppm, rank, n_buf, per_head, chunk_n, n_b,
                                          n_lowrank):
    w = gw.Workload("emu", B=B, H_kv=H, H_q=Hq, n=n, bits=bits, group=g, outlier_ppm=ppm, rank=rank,
                    rank_chunk=2, n_b=n_b, steps=1, seed=5)
    d = str(tmp_path)
    a = lambda t: t.numpy()
    oc = go.OracleCache(B, H, Hq, 128, bits, g, ppm, per_head)
    K, V, ib = a(gw.make_keys(w, n, 0)), a(gw.make_values(w, n, 0)), a(gw.make_init_B(w, rank, 0))
    for name, x in (("K", K), ("V", V), ("ib", ib)):
        x.tofile(os.path.join(d, name + ".bin"))
    if n_lowrank >= 0:
        oc.compress(K, V, rank, 3, ib, n_lowrank=n_lowrank)
    else:
        oc.compress(K, V, rank, 3, ib)
    Kc, Vc, ibc = a(gw.make_keys(w, chunk_n, 1)), a(gw.make_values(w, chunk_n, 1)), a(gw.make_init_B(w, 2, 1))
    for name, x in (("Kc0", Kc), ("Vc0", Vc), ("ibc0", ibc)):
        x.tofile(os.path.join(d, name + ".bin"))
    oc.compress(Kc, Vc, 2, 3, ibc)
    q, Kb, Vb = a(gw.make_queries(w, 0)), a(gw.make_keys(w, n_b, 50)), a(gw.make_values(w, n_b, 50))
    for name, x in (("q", q), ("Kb", Kb), ("Vb", Vb)):
        x.tofile(os.path.join(d, name + ".bin"))
    q2 = np.stack([q[:, :, 0], a(gw.make_queries(w, 1))[:, :, 0]], axis=2)       # two query rows per head
    q2.tofile(os.path.join(d, "q2.bin"))
    with open(os.path.join(d, "meta.txt"), "w") as f:
        f.write(" ".join(str(x) for x in [B, H, Hq, bits, g, ppm, n, rank, 1, chunk_n, 2, n_buf, n_b, 3, 1 if per_head else 0, n_lowrank]) + "\n")
    r = subprocess.run([emulator, d], capture_output=True, text=True, timeout=900,
                       env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
    assert r.returncode == 0, r.stderr[-4000:]
    assert "AddressSanitizer" not in r.stderr
    out = np.fromfile(os.path.join(d, "out.bin"), np.float16).reshape(B, Hq, 1, 128)
    oc.decode_attn(q, Kb, Vb, n_buf)
    pu.check_attention(out, oc.last_attn_f64)
    Ko, Vo = oc.decompress()
    Kg = np.fromfile(os.path.join(d, "Khat.bin"), np.float16).reshape(Ko.shape).astype(np.float64)
    Vg = np.fromfile(os.path.join(d, "Vhat.bin"), np.float16).reshape(Vo.shape).astype(np.float64)
    for got, want in ((Kg, Ko.astype(np.float64)), (Vg, Vo.astype(np.float64))):
        assert np.linalg.norm(got - want) <= 1e-3 * np.linalg.norm(want)
    # codes, scales and zero-points bit for bit, although this build lets the compiler contract
    for name, segs in (("K", oc.K), ("V", oc.V)):
        o_codes = np.concatenate([s.codes for s in segs], axis=2)
        o_scale = np.concatenate([s.scale for s in segs], axis=2)
        o_zero = np.concatenate([s.zero for s in segs], axis=2)
        codes = np.fromfile(os.path.join(d, name + "codes.bin"), np.uint8).reshape(o_codes.shape)
        scale = np.fromfile(os.path.join(d, name + "scale.bin"), np.float16).reshape(o_scale.shape)
        zero = np.fromfile(os.path.join(d, name + "zero.bin"), np.float16).reshape(o_zero.shape)
        assert np.array_equal(scale.view(np.uint16), o_scale.view(np.uint16)), name
        assert np.array_equal(zero.astype(np.float32), o_zero.astype(np.float32)), name
        assert np.array_equal(codes, o_codes), name
        # the sparse matrix: support and values bit for bit, as a dense view and in coordinate form
        o_mask = np.concatenate([s.mask for s in segs], axis=2)
        o_vals = np.concatenate([s.svals for s in segs], axis=2)
        mask = np.fromfile(os.path.join(d, name + "mask.bin"), np.uint8).reshape(o_mask.shape).astype(bool)
        vals = np.fromfile(os.path.join(d, name + "svals.bin"), np.uint16).reshape(o_mask.shape)
        assert np.array_equal(mask, o_mask), name
        assert np.array_equal(vals[o_mask], o_vals.view(np.uint16)[o_mask]) and not vals[~o_mask].any(), name
        want = np.flatnonzero(o_mask)
        assert np.array_equal(np.fromfile(os.path.join(d, name + "coo_idx.bin"), np.int64), want), name
        assert np.array_equal(np.fromfile(os.path.join(d, name + "coo_val.bin"), np.uint16),
                              o_vals.view(np.uint16).reshape(-1)[want]), name
    # the exported factors of the prefill segment give the oracle's low-rank product (bar of the GPU tests)
    if rank > 0:
        for name, seg in (("K", oc.K[0]), ("V", oc.V[0])):
            A = np.fromfile(os.path.join(d, name + "_A.bin"), np.float16).reshape(B, H, n, rank).astype(np.float64)
            Bf = np.fromfile(os.path.join(d, name + "_B.bin"), np.float16).reshape(B, H, 128, rank).astype(np.float64)
            got = A @ np.swapaxes(Bf, -1, -2)
            want = seg.A.astype(np.float64) @ np.swapaxes(seg.Bf.astype(np.float64), -1, -2)
            assert np.linalg.norm(got - want) <= pu.LOWRANK_REL_TOL * np.linalg.norm(want), name
    if 2 * (Hq // H) <= 8 and n_buf >= 2:
        out2 = np.fromfile(os.path.join(d, "out2.bin"), np.float16).reshape(B, Hq, 2, 128)
        pu.check_attention(out2, go.decode_attn_multi(oc, q2, Kb, Vb, n_buf, True), "two query rows")
