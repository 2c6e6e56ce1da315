"""ctypes binding of libsa_prefill.so: argument marshalling only.

Every step of the path runs in the HIP library; PyTorch is used for device
memory and streams.  The library must be present: nothing here falls back to
another implementation.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsa_prefill.so")

SA_PATTERN_AUTO, SA_TRIANGULAR, SA_INTERVAL_SLASH, SA_BLOCK_CLUSTER = -1, 0, 1, 2
_STATUS = {0: "SA_OK", 1: "SA_ERR_INVALID_ARG", 2: "SA_ERR_UNSUPPORTED",
           3: "SA_ERR_BUFFER_TOO_SMALL", 4: "SA_ERR_HIP"}


class SaError(RuntimeError):
    def __init__(self, status, msg=""):
        super().__init__(f"{_STATUS.get(status, status)} {msg}".strip())
        self.status = status


class SaConfig(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("seq_len", C.c_int32), ("block", C.c_int32), ("last_q", C.c_int32),
                ("softmax_scale", C.c_float),
                ("sink_blocks", C.c_int32), ("local_blocks", C.c_int32),
                ("k_vertical", C.c_int32), ("k_slash", C.c_int32), ("k_blocks", C.c_int32),
                ("probe_v", C.c_int32), ("probe_s", C.c_int32), ("lift_num", C.c_int32),
                ("lift_den", C.c_int32),
                ("q_head_stride", C.c_int64), ("q_row_stride", C.c_int64),
                ("kv_head_stride", C.c_int64), ("kv_row_stride", C.c_int64),
                ("block_select", C.c_int32), ("diagonal_select", C.c_int32),
                ("lazy_block_map", C.c_int32)]


class SaScores(C.Structure):
    _fields_ = [("v", C.c_void_p), ("s", C.c_void_p), ("blk", C.c_void_p)]


class SaIndex(C.Structure):
    _fields_ = [("pattern", C.c_void_p), ("n_cols", C.c_void_p), ("cols", C.c_void_p),
                ("n_offs", C.c_void_p), ("offs", C.c_void_p), ("rowptr", C.c_void_p),
                ("blkcols", C.c_void_p)]


_lib = None


def library():
    """Load libsa_prefill.so (built by paper_2412_06198_amd.build); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SaError(4, f"{LIB_PATH} is missing: run `python -m paper_2412_06198_amd.build`")
        lib = C.CDLL(LIB_PATH)
        vp, st = C.c_void_p, C.c_int
        lib.sa_version.restype = C.c_char_p
        lib.sa_last_error.restype = C.c_char_p
        lib.sa_last_error.argtypes = [vp]
        lib.sa_default_budgets.argtypes = [C.POINTER(SaConfig), C.c_double]
        lib.sa_create.argtypes = [C.POINTER(SaConfig), C.POINTER(vp)]
        lib.sa_destroy.argtypes = [vp]
        lib.sa_destroy.restype = None
        lib.sa_scores_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
        lib.sa_index_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
        lib.sa_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
        lib.sa_set_workspace.argtypes = [vp, vp, C.c_size_t]
        lib.sa_estimate_patterns.argtypes = [vp, vp, vp, SaScores, vp]
        lib.sa_build_index.argtypes = [vp, SaScores, C.POINTER(C.c_int32), SaIndex, vp]
        lib.sa_estimate_and_index.argtypes = [vp, vp, vp, SaScores, C.POINTER(C.c_int32), SaIndex, vp]
        lib.sa_sparse_prefill.argtypes = [vp, vp, vp, vp, SaIndex, vp, vp]
        lib.sa_sparse_prefill_counted.argtypes = [vp, vp, vp, vp, SaIndex, vp, vp, vp]
        lib.sa_sparse_decode.argtypes = [vp, vp, vp, vp, SaIndex, C.c_int64, vp, vp]
        lib.sa_sparse_decode_static.argtypes = [vp, vp, vp, vp, SaIndex, C.c_int64, vp, vp]
        lib.sa_search_scratch_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
        lib.sa_search_patterns.argtypes = [vp, vp, vp, vp, SaScores, C.c_int64, C.c_int64, vp, C.c_size_t,
                                           C.POINTER(SaSearchHead), vp]
        for f in ("sa_default_budgets", "sa_create", "sa_scores_bytes", "sa_index_bytes",
                  "sa_workspace_bytes", "sa_set_workspace", "sa_estimate_patterns",
                  "sa_build_index", "sa_sparse_prefill", "sa_sparse_prefill_counted",
                  "sa_search_scratch_bytes", "sa_search_patterns", "sa_sparse_decode",
                  "sa_sparse_decode_static", "sa_estimate_and_index"):
            getattr(lib, f).restype = st
        _lib = lib
    return _lib


def _ptr(x):
    """Device address of a torch tensor, or an int passed through."""
    if x is None:
        return None
    return x if isinstance(x, int) else x.data_ptr()


def _check(status, ctx=None):
    if status != 0:
        msg = library().sa_last_error(ctx).decode() if ctx else ""
        raise SaError(status, msg)


def sa_version() -> str:
    return library().sa_version().decode()


def sa_last_error(ctx) -> str:
    return library().sa_last_error(ctx).decode()


def sa_default_budgets(cfg: SaConfig, keep_fraction: float) -> SaConfig:
    _check(library().sa_default_budgets(C.byref(cfg), keep_fraction))
    return cfg


def sa_create(cfg: SaConfig):
    ctx = C.c_void_p()
    _check(library().sa_create(C.byref(cfg), C.byref(ctx)))
    return ctx


def sa_destroy(ctx):
    library().sa_destroy(ctx)


def sa_scores_bytes(ctx):
    out = (C.c_size_t * 3)()
    _check(library().sa_scores_bytes(ctx, out), ctx)
    return list(out)


def sa_index_bytes(ctx):
    out = (C.c_size_t * 7)()
    _check(library().sa_index_bytes(ctx, out), ctx)
    return list(out)


def sa_workspace_bytes(ctx) -> int:
    out = C.c_size_t()
    _check(library().sa_workspace_bytes(ctx, C.byref(out)), ctx)
    return out.value


def sa_set_workspace(ctx, dev, nbytes):
    _check(library().sa_set_workspace(ctx, _ptr(dev), nbytes), ctx)


def sa_estimate_patterns(ctx, Q, K, scores: SaScores, stream=None):
    _check(library().sa_estimate_patterns(ctx, _ptr(Q), _ptr(K), scores, stream), ctx)


def _override_array(pattern_override, n_q_heads):
    """Host int32 array of exactly n_q_heads entries (the library reads that many), or None."""
    if pattern_override is None:
        return None
    if n_q_heads is None or len(pattern_override) != n_q_heads:
        raise SaError(1, f"pattern_override needs one entry per query head ({n_q_heads}), got {len(pattern_override)}")
    return (C.c_int32 * n_q_heads)(*[int(p) for p in pattern_override])


def sa_build_index(ctx, scores: SaScores, pattern_override, index: SaIndex, stream=None, n_q_heads=None):
    ov = _override_array(pattern_override, n_q_heads)
    _check(library().sa_build_index(ctx, scores, ov, index, stream), ctx)


def sa_estimate_and_index(ctx, Q, K, scores: SaScores, pattern_override, index: SaIndex, stream=None,
                          n_q_heads=None):
    ov = _override_array(pattern_override, n_q_heads)
    _check(library().sa_estimate_and_index(ctx, _ptr(Q), _ptr(K), scores, ov, index, stream), ctx)


def sa_sparse_prefill(ctx, Q, K, V, index: SaIndex, O, stream=None):
    _check(library().sa_sparse_prefill(ctx, _ptr(Q), _ptr(K), _ptr(V), index, _ptr(O), stream), ctx)


def sa_sparse_prefill_counted(ctx, Q, K, V, index: SaIndex, O, counters, stream=None):
    _check(library().sa_sparse_prefill_counted(ctx, _ptr(Q), _ptr(K), _ptr(V), index, _ptr(O),
                                               _ptr(counters), stream), ctx)


def sa_sparse_decode(ctx, q, K, V, index: SaIndex, pos, o, stream=None):
    _check(library().sa_sparse_decode(ctx, _ptr(q), _ptr(K), _ptr(V), index, C.c_int64(int(pos)), _ptr(o), stream), ctx)


def sa_sparse_decode_static(ctx, q, K, V, index: SaIndex, pos, o, stream=None):
    _check(library().sa_sparse_decode_static(ctx, _ptr(q), _ptr(K), _ptr(V), index, C.c_int64(int(pos)), _ptr(o),
                                             stream), ctx)


class SaSearchHead(C.Structure):
    _fields_ = [("pattern", C.c_int32), ("param", C.c_int32 * 3), ("pairs", C.c_int64 * 3),
                ("err", C.c_double * 3)]


def sa_search_scratch_bytes(ctx) -> int:
    out = C.c_size_t()
    _check(library().sa_search_scratch_bytes(ctx, C.byref(out)), ctx)
    return out.value


def sa_search_patterns(ctx, Q, K, V, scores: SaScores, target_pairs, eps_pairs, scratch, scratch_bytes,
                       n_heads, stream=None):
    out = (SaSearchHead * n_heads)()
    _check(library().sa_search_patterns(ctx, _ptr(Q), _ptr(K), _ptr(V), scores, C.c_int64(int(target_pairs)),
                                        C.c_int64(int(eps_pairs)), _ptr(scratch), C.c_size_t(scratch_bytes),
                                        out, stream), ctx)
    return [{"pattern": int(r.pattern), "param": list(r.param), "pairs": list(r.pairs), "err": list(r.err)}
            for r in out]


class Session:
    """Owns a context plus the torch-allocated score / index / workspace buffers of one shape."""

    def __init__(self, n_q_heads, n_kv_heads, seq_len, block, last_q, keep=None, device="cuda:0",
                 **budgets):
        import torch

        self.torch = torch
        self.device = torch.device(device)
        cfg = SaConfig()
        cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim = n_q_heads, n_kv_heads, 128
        cfg.seq_len, cfg.block, cfg.last_q = seq_len, block, last_q
        if keep is not None:
            sa_default_budgets(cfg, keep)
        for k, v in budgets.items():
            setattr(cfg, k, v)
        self.cfg = cfg
        self.ctx = sa_create(cfg)
        i32, f32 = torch.int32, torch.float32
        sb = sa_scores_bytes(self.ctx)
        ib = sa_index_bytes(self.ctx)
        H, N, nb = n_q_heads, seq_len, seq_len // block
        dev = self.device
        self.v = torch.empty((H, N), dtype=f32, device=dev)
        self.s = torch.empty((H, N), dtype=f32, device=dev)
        self.blk = torch.empty((H, nb, nb), dtype=f32, device=dev)
        assert [self.v.nbytes, self.s.nbytes, self.blk.nbytes] == sb
        self.cap_b = ib[6] // (4 * H)
        self.pattern = torch.empty(H, dtype=i32, device=dev)
        self.n_cols = torch.empty(H, dtype=i32, device=dev)
        self.cols = torch.empty((H, cfg.k_vertical), dtype=i32, device=dev)
        self.n_offs = torch.empty(H, dtype=i32, device=dev)
        self.offs = torch.empty((H, cfg.k_slash), dtype=i32, device=dev)
        self.rowptr = torch.empty((H, nb + 1), dtype=i32, device=dev)
        self.blkcols = torch.empty((H, self.cap_b), dtype=i32, device=dev)
        assert [t.nbytes for t in self.index_tensors()] == ib
        self.ws = torch.empty(sa_workspace_bytes(self.ctx) + 256, dtype=torch.uint8, device=dev)
        off = (-self.ws.data_ptr()) % 256
        sa_set_workspace(self.ctx, self.ws.data_ptr() + off, self.ws.nbytes - off)

    def index_tensors(self):
        return [self.pattern, self.n_cols, self.cols, self.n_offs, self.offs, self.rowptr,
                self.blkcols]

    def scores(self) -> SaScores:
        return SaScores(self.v.data_ptr(), self.s.data_ptr(), self.blk.data_ptr())

    def index(self) -> SaIndex:
        return SaIndex(*[t.data_ptr() for t in self.index_tensors()])

    def stream(self):
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def estimate(self, Q, K):
        sa_estimate_patterns(self.ctx, Q, K, self.scores(), self.stream())

    def build_index(self, pattern_override=None):
        sa_build_index(self.ctx, self.scores(), pattern_override, self.index(), self.stream(),
                       n_q_heads=self.cfg.n_q_heads)

    def estimate_and_index(self, Q, K, pattern_override=None):
        sa_estimate_and_index(self.ctx, Q, K, self.scores(), pattern_override, self.index(), self.stream(),
                              n_q_heads=self.cfg.n_q_heads)

    def prefill(self, Q, K, V, O):
        sa_sparse_prefill(self.ctx, Q, K, V, self.index(), O, self.stream())

    def prefill_counted(self, Q, K, V, O):
        """Returns (32x32 sub-tiles multiplied, kept query-key pairs) of one prefill call."""
        cnt = self.torch.zeros(2, dtype=self.torch.int64, device=self.device)
        sa_sparse_prefill_counted(self.ctx, Q, K, V, self.index(), O, cnt, self.stream())
        self.torch.cuda.synchronize(self.device)
        return [int(x) for x in cnt.cpu()]

    def decode(self, q, K, V, pos, o):
        """One decode step at position pos >= seq_len over the current index."""
        sa_sparse_decode(self.ctx, q, K, V, self.index(), pos, o, self.stream())

    def decode_static(self, q, K, V, pos, o):
        """The same step through the entry point that keeps its partial results in the library's
        static device array (no workspace needed, nothing allocated)."""
        sa_sparse_decode_static(self.ctx, q, K, V, self.index(), pos, o, self.stream())

    def search_patterns(self, Q, K, V, target_pairs, eps_pairs):
        """Alg. 1 on the scores of the last estimate(): one dict per head."""
        nbytes = sa_search_scratch_bytes(self.ctx)
        scratch = self.torch.empty(nbytes + 256, dtype=self.torch.uint8, device=self.device)
        off = (-scratch.data_ptr()) % 256
        return sa_search_patterns(self.ctx, Q, K, V, self.scores(), target_pairs, eps_pairs,
                                  scratch.data_ptr() + off, nbytes, self.cfg.n_q_heads, self.stream())

    def close(self):
        if self.ctx is not None:
            sa_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
