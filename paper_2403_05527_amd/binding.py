"""ctypes binding of libgear (include/gear.h).  Argument marshalling only: every
step of the path runs in the HIP library; torch supplies device memory and the
current stream.  There is no CPU fallback: a missing library is an error."""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libgear.so")

GEAR_MAX_CHUNKS = 256
GEAR_STATIC_SCRATCH_BYTES = 32 << 20
GEAR_OK, GEAR_EINVAL, GEAR_ECAPACITY, GEAR_EALIGN, GEAR_EHIP = 0, -1, -2, -3, -4

EXPORTED = [
    "gear_cache_bytes", "gear_cache_init", "gear_cache_reset", "gear_compress", "gear_compress_recent", "gear_decompress",
    "gear_decode_attn", "gear_decode_attn_mq", "gear_decode_attn_static", "gear_export_codes", "gear_export_sparse", "gear_export_sparse_coo", "gear_export_lowrank", "gear_strerror",
]


class gear_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "B", "H_kv", "H_q", "d_h", "bits", "group", "outlier_ppm", "n_buf_cap", "n_prefill_max",
        "n_chunks_max", "rank_max", "flags")]


class gear_cache(ctypes.Structure):
    _fields_ = [
        ("cfg", gear_config),
        ("arena", ctypes.c_void_p),
        ("arena_bytes", ctypes.c_uint64),
        ("n_prefill", ctypes.c_int32),
        ("rank_prefill", ctypes.c_int32),
        ("n_chunks", ctypes.c_int32),
        ("n_total", ctypes.c_int32),
        ("chunk_n", ctypes.c_uint8 * GEAR_MAX_CHUNKS),
        ("chunk_rank", ctypes.c_uint8 * GEAR_MAX_CHUNKS),
    ]


class GearError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (what, strerror(status), status))


_lib = None


def load_library():
    """Loads libgear.so built in-tree (python -m paper_2403_05527_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libgear.so is not built (%s); run __graft_entry__.build()" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    cfgp, cachep = ctypes.POINTER(gear_config), ctypes.POINTER(gear_cache)
    lib.gear_cache_bytes.argtypes = [cfgp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.gear_cache_init.argtypes = [cfgp, vp, sz, cachep]
    lib.gear_cache_reset.argtypes = [cachep]
    lib.gear_compress.argtypes = [cachep, vp, vp, i32, i32, i32, vp, ctypes.c_uint64, vp, sz, vp]
    lib.gear_compress_recent.argtypes = [cachep, vp, vp, i32, i32, i32, vp, ctypes.c_uint64, i32, vp, sz, vp]
    lib.gear_decompress.argtypes = [cachep, vp, vp, vp]
    lib.gear_decode_attn.argtypes = [cachep, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.gear_decode_attn_mq.argtypes = [cachep, vp, i32, i32, vp, vp, i32, vp, vp, sz, vp]
    lib.gear_decode_attn_static.argtypes = [cachep, vp, vp, vp, i32, vp, vp]
    lib.gear_export_codes.argtypes = [cachep, ctypes.c_int, vp, vp, vp, vp]
    lib.gear_export_sparse.argtypes = [cachep, ctypes.c_int, vp, vp, vp]
    lib.gear_export_sparse_coo.argtypes = [cachep, ctypes.c_int, ctypes.POINTER(ctypes.c_int64), vp, vp, vp, sz, vp]
    lib.gear_export_lowrank.argtypes = [cachep, ctypes.c_int, ctypes.c_int, vp, vp, vp]
    lib.gear_strerror.argtypes = [ctypes.c_int]
    lib.gear_strerror.restype = ctypes.c_char_p
    for name in EXPORTED:
        if name != "gear_strerror":
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(status):
    return load_library().gear_strerror(int(status)).decode()


def _check(status, what):
    if status != GEAR_OK:
        raise GearError(status, what)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


GEAR_FLAG_V_FILTER_PER_HEAD = 1


def make_config(B, H_kv, H_q, bits, group, outlier_ppm, n_buf_cap, n_prefill_max, n_chunks_max, rank_max,
                d_h=128, flags=0):
    return gear_config(B, H_kv, H_q, d_h, bits, group, outlier_ppm, n_buf_cap, n_prefill_max, n_chunks_max,
                       rank_max, flags)


# ---- thin wrappers with the C names ---------------------------------------
def gear_cache_bytes(cfg):
    a, w = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(load_library().gear_cache_bytes(ctypes.byref(cfg), ctypes.byref(a), ctypes.byref(w)), "gear_cache_bytes")
    return a.value, w.value


def gear_cache_init(cfg, arena):
    cache = gear_cache()
    _check(load_library().gear_cache_init(ctypes.byref(cfg), _ptr(arena), arena.numel() * arena.element_size(),
                                          ctypes.byref(cache)), "gear_cache_init")
    return cache


def gear_cache_reset(cache):
    _check(load_library().gear_cache_reset(ctypes.byref(cache)), "gear_cache_reset")


def gear_compress(cache, K, V, rank, iters, init_B, workspace, seed=0):
    n = K.shape[2]
    _check(load_library().gear_compress(ctypes.byref(cache), _ptr(K), _ptr(V), n, rank, iters, _ptr(init_B),
                                        ctypes.c_uint64(seed), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "gear_compress")


def gear_compress_recent(cache, K, V, rank, iters, init_B, n_lowrank, workspace, seed=0):
    n = K.shape[2]
    _check(load_library().gear_compress_recent(ctypes.byref(cache), _ptr(K), _ptr(V), n, rank, iters, _ptr(init_B),
                                               ctypes.c_uint64(seed), n_lowrank, _ptr(workspace),
                                               workspace.numel() * workspace.element_size(), _stream()),
           "gear_compress_recent")


def gear_decompress(cache, K_out, V_out):
    _check(load_library().gear_decompress(ctypes.byref(cache), _ptr(K_out), _ptr(V_out), _stream()),
           "gear_decompress")


def gear_decode_attn(cache, q, K_buf, V_buf, n_buf, out, workspace):
    _check(load_library().gear_decode_attn(ctypes.byref(cache), _ptr(q), _ptr(K_buf), _ptr(V_buf), n_buf, _ptr(out),
                                           _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "gear_decode_attn")


def gear_decode_attn_mq(cache, q, causal, K_buf, V_buf, n_buf, out, workspace):
    _check(load_library().gear_decode_attn_mq(ctypes.byref(cache), _ptr(q), q.shape[2], 1 if causal else 0, _ptr(K_buf),
                                              _ptr(V_buf), n_buf, _ptr(out), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream()),
           "gear_decode_attn_mq")


def gear_decode_attn_static(cache, q, K_buf, V_buf, n_buf, out):
    _check(load_library().gear_decode_attn_static(ctypes.byref(cache), _ptr(q), _ptr(K_buf), _ptr(V_buf), n_buf,
                                                  _ptr(out), _stream()), "gear_decode_attn_static")


def gear_export_codes(cache, which, codes, scale, zero):
    _check(load_library().gear_export_codes(ctypes.byref(cache), which, _ptr(codes), _ptr(scale), _ptr(zero),
                                            _stream()), "gear_export_codes")


def gear_export_sparse(cache, which, mask, values):
    _check(load_library().gear_export_sparse(ctypes.byref(cache), which, _ptr(mask), _ptr(values), _stream()),
           "gear_export_sparse")


def gear_export_sparse_coo(cache, which, lin_index, values, workspace):
    """Returns nnz; with lin_index = values = None only the count is computed (nothing is launched)."""
    nnz = ctypes.c_int64(0)
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().gear_export_sparse_coo(ctypes.byref(cache), which, ctypes.byref(nnz), _ptr(lin_index),
                                                 _ptr(values), _ptr(workspace), wb, _stream()), "gear_export_sparse_coo")
    return nnz.value


def gear_export_lowrank(cache, which, seg, A, Bf):
    _check(load_library().gear_export_lowrank(ctypes.byref(cache), which, seg, _ptr(A), _ptr(Bf), _stream()),
           "gear_export_lowrank")


# ---- convenience owner of the device buffers -------------------------------
class GearCache:
    """Allocates the arena and workspace with torch and forwards to the C ABI."""

    def __init__(self, cfg, device="cuda:0"):
        self.cfg = cfg
        self.device = torch.device(device)
        a, w = gear_cache_bytes(cfg)
        self.arena_bytes, self.workspace_bytes = a, w
        self.arena = torch.empty(a, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(w, dtype=torch.uint8, device=self.device)
        self.cache = gear_cache_init(cfg, self.arena)

    @property
    def n_total(self):
        return self.cache.n_total

    def n_groups_total(self):
        g = self.cfg.group
        if g == 0:                                  # per-vector groups: one Key group per segment
            return (1 if self.cache.n_prefill > 0 else 0) + self.cache.n_chunks
        ng = -(-self.cache.n_prefill // g)
        for j in range(self.cache.n_chunks):
            ng += -(-self.cache.chunk_n[j] // g)
        return ng

    def reset(self):
        gear_cache_reset(self.cache)

    def compress(self, K, V, rank, iters=3, init_B=None, seed=0, n_lowrank=None):
        if n_lowrank is None:
            gear_compress(self.cache, K, V, rank, iters, init_B, self.workspace, seed)
        else:
            gear_compress_recent(self.cache, K, V, rank, iters, init_B, n_lowrank, self.workspace, seed)

    def decompress(self):
        c = self.cfg
        shape = (c.B, c.H_kv, self.n_total, c.d_h)
        K = torch.empty(shape, dtype=torch.float16, device=self.device)
        V = torch.empty(shape, dtype=torch.float16, device=self.device)
        gear_decompress(self.cache, K, V)
        return K, V

    def decode_attn(self, q, K_buf=None, V_buf=None, n_buf=0, out=None):
        if out is None:
            out = torch.empty_like(q)
        gear_decode_attn(self.cache, q, K_buf, V_buf, n_buf, out, self.workspace)
        return out

    def decode_attn_mq(self, q, K_buf, V_buf, n_buf, causal=True, out=None):
        if out is None:
            out = torch.empty_like(q)
        gear_decode_attn_mq(self.cache, q, causal, K_buf, V_buf, n_buf, out, self.workspace)
        return out

    def export_codes(self, which):
        c = self.cfg
        codes = torch.empty((c.B, c.H_kv, self.n_total, c.d_h), dtype=torch.uint8, device=self.device)
        if which == 0:
            shape = (c.B, c.H_kv, self.n_groups_total(), c.d_h)
        else:
            shape = (c.B, c.H_kv, self.n_total, c.d_h // (c.group or c.d_h))
        scale = torch.empty(shape, dtype=torch.float16, device=self.device)
        zero = torch.empty(shape, dtype=torch.float16, device=self.device)
        gear_export_codes(self.cache, which, codes, scale, zero)
        return codes, scale, zero

    def export_sparse(self, which):
        c = self.cfg
        shape = (c.B, c.H_kv, self.n_total, c.d_h)
        mask = torch.empty(shape, dtype=torch.uint8, device=self.device)
        vals = torch.empty(shape, dtype=torch.float16, device=self.device)
        gear_export_sparse(self.cache, which, mask, vals)
        return mask, vals

    def export_sparse_coo(self, which):
        nnz = gear_export_sparse_coo(self.cache, which, None, None, None)
        lin = torch.empty(max(nnz, 1), dtype=torch.int64, device=self.device)
        vals = torch.empty(max(nnz, 1), dtype=torch.float16, device=self.device)
        gear_export_sparse_coo(self.cache, which, lin, vals, self.workspace)
        return lin[:nnz], vals[:nnz]

    def export_lowrank(self, which, seg):
        c = self.cfg
        n = self.cache.n_prefill if seg == 0 else self.cache.chunk_n[seg - 1]
        r = self.cache.rank_prefill if seg == 0 else self.cache.chunk_rank[seg - 1]
        A = torch.empty((c.B, c.H_kv, n, r), dtype=torch.float16, device=self.device)
        Bf = torch.empty((c.B, c.H_kv, c.d_h, r), dtype=torch.float16, device=self.device)
        if r > 0:
            gear_export_lowrank(self.cache, which, seg, A, Bf)
        return A, Bf
