"""ctypes binding of the C ABI in include/distshap.h.

Every method of `Context` is one call of the function of the same name
(`Context.explain` -> `ds_explain`, ...): it only allocates output tensors,
passes device pointers, and turns a non-zero status into `DistShapError`.
There is no fallback: without the built library every call raises.
"""
import ctypes as C
import os

DS_OK, DS_EINVAL, DS_ECAPACITY, DS_ENOMEM, DS_ENOTCONV, DS_EDEVICE, DS_ESINGULAR, DS_EINTERNAL = range(8)
DS_F32, DS_BF16_IN_F32_ACC = 0, 1
DS_SCORE_PROB, DS_SCORE_LOGIT = 0, 1
DS_SOLVER_AUTO, DS_SOLVER_GRAM_CHOL, DS_SOLVER_CGLS = 0, 1, 2
DS_WEIGHT_CLASS_MASS, DS_WEIGHT_UNIFORM = 0, 1

EXPORTED_SYMBOLS = [
    "ds_create", "ds_destroy", "ds_last_error", "ds_set_tuning", "ds_set_graph", "ds_set_features", "ds_set_gcn", "ds_set_gat",
    "ds_explain", "ds_explain_batch", "ds_extract", "ds_cgraph_get_info", "ds_cgraph_edges",
    "ds_cgraph_nodes", "ds_cgraph_first_transform", "ds_cgraph_free", "ds_sample_plan", "ds_sample",
    "ds_plan_tables", "ds_plan_tables_ex", "ds_sample_ex", "ds_sample_range", "ds_eval", "ds_eval_pairs", "ds_eval_noalloc", "ds_solve", "ds_fidelity", "ds_copy_probe", "ds_version",
]


class Options(C.Structure):
    _fields_ = [("hops", C.c_int32), ("directed", C.c_int32), ("score", C.c_int32),
                ("solver", C.c_int32), ("tol", C.c_double), ("max_iter", C.c_int32),
                ("batch_rows", C.c_int32), ("paired", C.c_int32), ("weighting", C.c_int32),
                ("saturate", C.c_int32)]


class Tuning(C.Structure):
    _fields_ = [("batch_workers", C.c_int32), ("gram_sparse_div", C.c_int32), ("gram_dense_fraction", C.c_float),
                ("sampler_window", C.c_int32), ("eval_path", C.c_int32), ("cgls_dense_div", C.c_int32),
                ("pair_lists", C.c_int32)]


class Report(C.Structure):
    _fields_ = [("num_players", C.c_int64), ("num_nodes", C.c_int64), ("num_entries", C.c_int64),
                ("num_rows", C.c_int64), ("enumerated", C.c_int32), ("pred_class", C.c_int32),
                ("solver_used", C.c_int32), ("cgls_iterations", C.c_int32),
                ("cgls_rel_residual", C.c_double), ("f_empty", C.c_double), ("f_full", C.c_double),
                ("ms_extract", C.c_float), ("ms_sample", C.c_float), ("ms_eval", C.c_float),
                ("ms_solve", C.c_float), ("ms_total", C.c_float),
                ("ms_k_eval", C.c_float), ("ms_k_gram", C.c_float), ("ms_k_chol", C.c_float),
                ("ms_k_cgls", C.c_float),
                ("num_pairs", C.c_int64), ("bytes_sample", C.c_double), ("bytes_eval", C.c_double),
                ("bytes_solve", C.c_double), ("ms_k_stream", C.c_float)]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


class CGraphInfo(C.Structure):
    _fields_ = [("num_players", C.c_int64), ("num_nodes", C.c_int64), ("num_entries", C.c_int64),
                ("target", C.c_int64), ("hops", C.c_int32), ("directed", C.c_int32),
                ("ball", C.c_int64 * 8)]


class DistShapError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"distshap status {code}: {message}")
        self.code = code


def library_path():
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdistshap_hip.so")


_lib = None


def load_library():
    """Load the built library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime: it has to be the one already in the process when this
    # library (linked against libamdhip64) is loaded, or two runtimes end up side by side
    import torch  # noqa: F401
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python -m paper_2506_22668_amd.build` first")
    lib = C.CDLL(path)
    p, i32, i64, u64, u32, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_uint32, C.c_double
    sigs = {
        "ds_create": [C.POINTER(p), C.c_int, p],
        "ds_destroy": [p],
        "ds_set_tuning": [p, C.POINTER(Tuning)],
        "ds_set_graph": [p, i64, p, p],
        "ds_set_features": [p, p, i32, i32],
        "ds_set_gcn": [p, i32, C.POINTER(i32), C.POINTER(p), C.POINTER(p), i32],
        "ds_set_gat": [p, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(p), C.POINTER(p), C.POINTER(p), C.POINTER(p),
                       C.c_float],
        "ds_explain": [p, i64, i64, u64, C.POINTER(Options), p, C.POINTER(i64), p, p, C.POINTER(Report)],
        "ds_explain_batch": [p, C.POINTER(i64), i32, i64, u64, C.POINTER(Options), p, C.POINTER(i64),
                             C.POINTER(i64), p, p, i64, C.POINTER(Report)],
        "ds_extract": [p, i64, C.POINTER(Options), C.POINTER(p)],
        "ds_cgraph_get_info": [p, C.POINTER(CGraphInfo)],
        "ds_cgraph_edges": [p, p, p, p],
        "ds_cgraph_nodes": [p, p, p, p],
        "ds_cgraph_first_transform": [p, p, p],
        "ds_cgraph_free": [p, p],
        "ds_sample_plan": [i64, i64, C.POINTER(i64), C.POINTER(i32)],
        "ds_sample": [p, i64, i64, u64, u32, p, p, p, C.POINTER(i64)],
        "ds_plan_tables": [i64, i64, p, p],
        "ds_plan_tables_ex": [i64, i64, C.POINTER(Options), p, p, C.POINTER(i64)],
        "ds_sample_ex": [p, i64, i64, u64, u32, C.POINTER(Options), p, p, p, C.POINTER(i64)],
        "ds_sample_range": [p, i64, i64, u64, u32, i64, i64, p, p, p],
        "ds_eval": [p, p, p, i64, i32, p, C.POINTER(i32)],
        "ds_eval_pairs": [p, p, p, i64, i32, p, C.POINTER(i32)],
        "ds_eval_noalloc": [p, p, p, i64, i32, p],
        "ds_solve": [p, i64, i64, p, p, p, C.POINTER(Options), p, C.POINTER(Report)],
        "ds_copy_probe": [p, p, p, i64],
        "ds_fidelity": [p, p, p, C.POINTER(i64), i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_float), p],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.ds_last_error.argtypes = [p]
    lib.ds_last_error.restype = C.c_char_p
    lib.ds_version.argtypes = []
    lib.ds_version.restype = C.c_char_p
    _lib = lib
    return lib


def sample_plan(n, n_samples):
    """(k, enumerated) for n players and a sample budget (host-only call)."""
    lib = load_library()
    k, e = C.c_int64(), C.c_int32()
    rc = lib.ds_sample_plan(n, n_samples, C.byref(k), C.byref(e))
    if rc != DS_OK:
        raise DistShapError(rc, "ds_sample_plan: bad arguments")
    return k.value, bool(e.value)


def plan_tables(n, n_samples, options=None):
    """(b int64[H+1], wtab float32[H+1]) of the sampling plan (host-only call); with `options` also the number of
    enumerated size classes (ds_plan_tables_ex)."""
    import numpy as np
    lib = load_library()
    H = n // 2
    b = np.zeros(H + 1, dtype=np.int64)
    wtab = np.zeros(H + 1, dtype=np.float32)
    if options is None:
        rc = lib.ds_plan_tables(n, n_samples, b.ctypes.data_as(C.c_void_p), wtab.ctypes.data_as(C.c_void_p))
        if rc != DS_OK:
            raise DistShapError(rc, "ds_plan_tables: bad arguments")
        return b, wtab
    upto = C.c_int64()
    rc = lib.ds_plan_tables_ex(n, n_samples, C.byref(options), b.ctypes.data_as(C.c_void_p),
                               wtab.ctypes.data_as(C.c_void_p), C.byref(upto))
    if rc != DS_OK:
        raise DistShapError(rc, "ds_plan_tables_ex: bad arguments")
    return b, wtab, upto.value


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


class Context:
    """One ds_ctx on a torch device; keeps the tensors registered with ds_set_* alive."""

    def __init__(self, device="cuda:0", stream=None):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.device = torch.device(device)
        idx = self.device.index if self.device.index is not None else 0
        self._stream = stream
        handle = C.c_void_p()
        sptr = C.c_void_p(stream.cuda_stream) if stream is not None else C.c_void_p(0)
        rc = self.lib.ds_create(C.byref(handle), idx, sptr)
        if rc != DS_OK:
            raise DistShapError(rc, "ds_create failed")
        self.h = handle
        self._keep = {}

    def close(self):
        if getattr(self, "h", None):
            self.lib.ds_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc, allow=()):
        if rc != DS_OK and rc not in allow:
            raise DistShapError(rc, self.lib.ds_last_error(self.h).decode())
        return rc

    def _sync_inputs(self):
        # inputs were produced on torch's current stream; the library runs on its own
        self.torch.cuda.current_stream(self.device).synchronize()

    def set_tuning(self, tuning=None):
        self._check(self.lib.ds_set_tuning(self.h, C.byref(tuning) if tuning is not None else None))

    # -- registration --------------------------------------------------------
    def set_graph(self, row_ptr, col):
        t = self.torch
        rp = t.as_tensor(row_ptr, dtype=t.int64).to(self.device).contiguous()
        ci = t.as_tensor(col, dtype=t.int32).to(self.device).contiguous()
        self._sync_inputs()
        self._check(self.lib.ds_set_graph(self.h, rp.numel() - 1, _ptr(rp), _ptr(ci)))
        self._keep["graph"] = (rp, ci)

    def set_features(self, X):
        t = self.torch
        X = t.as_tensor(X, dtype=t.float32).to(self.device).contiguous()
        self._sync_inputs()
        self._check(self.lib.ds_set_features(self.h, _ptr(X), X.shape[1], DS_F32))
        self._keep["X"] = X

    def set_gcn(self, weights, biases=None, transform_dtype=DS_F32):
        t = self.torch
        Ws = [t.as_tensor(w, dtype=t.float32).to(self.device).contiguous() for w in weights]
        L = len(Ws)
        dims = [Ws[0].shape[0]] + [w.shape[1] for w in Ws]
        Bs = None
        if biases is not None:
            Bs = [None if b is None else t.as_tensor(b, dtype=t.float32).to(self.device).contiguous() for b in biases]
        self._sync_inputs()
        dims_c = (C.c_int32 * (L + 1))(*dims)
        W_c = (C.c_void_p * L)(*[w.data_ptr() for w in Ws])
        B_c = None
        if Bs is not None:
            B_c = (C.c_void_p * L)(*[(b.data_ptr() if b is not None else 0) for b in Bs])
        self._check(self.lib.ds_set_gcn(self.h, L, dims_c, W_c, B_c, transform_dtype))
        self._keep["model"] = (Ws, Bs)
        self.dims = dims
        self.first_width = dims[1]

    def set_gat(self, weights, att_src, att_dst, heads, biases=None, negative_slope=0.2):
        """weights[l]: [in_l, heads_l * width_l]; att_src[l], att_dst[l]: [heads_l, width_l]."""
        t = self.torch
        dev = lambda a: t.as_tensor(a, dtype=t.float32).to(self.device).contiguous()
        Ws, As, Ad = [dev(w) for w in weights], [dev(a) for a in att_src], [dev(a) for a in att_dst]
        L = len(Ws)
        heads = [int(h) for h in heads]
        head_dims = [Ws[0].shape[0]] + [Ws[l].shape[1] // heads[l] for l in range(L)]
        Bs = None
        if biases is not None:
            Bs = [None if b is None else dev(b) for b in biases]
        self._sync_inputs()
        arr = lambda ts: (C.c_void_p * L)(*[(x.data_ptr() if x is not None else 0) for x in ts])
        self._check(self.lib.ds_set_gat(self.h, L, (C.c_int32 * (L + 1))(*head_dims), (C.c_int32 * L)(*heads),
                                        arr(Ws), arr(As), arr(Ad), None if Bs is None else arr(Bs),
                                        C.c_float(negative_slope)))
        self._keep["model"] = (Ws, As, Ad, Bs)
        self.dims = [head_dims[0]] + [heads[l] * head_dims[l + 1] for l in range(L - 1)] + [head_dims[L]]
        self.first_width = heads[0] * head_dims[1]

    # -- one-shot --------------------------------------------------------------
    def explain(self, target, n_samples, seed, options=None, capacity=None, want_edges=True,
                allow_not_converged=False):
        t = self.torch
        opts = options or Options()
        if capacity is None:
            cg = self.extract(target, opts)
            capacity = self.cgraph_info(cg).num_players
            self.cgraph_free(cg)
        cap = max(int(capacity), 1)
        phi = t.empty(cap, dtype=t.float32, device=self.device)
        es = t.empty(cap, dtype=t.int64, device=self.device) if want_edges else None
        ed = t.empty(cap, dtype=t.int64, device=self.device) if want_edges else None
        m = C.c_int64(int(capacity))
        rep = Report()
        self._sync_inputs()
        rc = self._check(self.lib.ds_explain(self.h, int(target), int(n_samples), C.c_uint64(int(seed)),
                                             C.byref(opts), _ptr(phi), C.byref(m), _ptr(es), _ptr(ed),
                                             C.byref(rep)),
                         allow=(DS_ENOTCONV,) if allow_not_converged else ())
        n = m.value
        return phi[:n], (es[:n] if want_edges else None), (ed[:n] if want_edges else None), rep, rc

    def explain_batch(self, targets, n_samples, seed, options=None, capacity=0):
        t = self.torch
        opts = options or Options()
        T = len(targets)
        cap = max(int(capacity), 1)
        phi = t.empty(cap, dtype=t.float32, device=self.device)
        es = t.empty(cap, dtype=t.int64, device=self.device)
        ed = t.empty(cap, dtype=t.int64, device=self.device)
        tg = (C.c_int64 * T)(*[int(x) for x in targets])
        M = (C.c_int64 * T)()
        off = (C.c_int64 * (T + 1))()
        reps = (Report * T)()
        self._sync_inputs()
        rc = self._check(self.lib.ds_explain_batch(self.h, tg, T, int(n_samples), C.c_uint64(int(seed)),
                                                   C.byref(opts), _ptr(phi), M, off, _ptr(es), _ptr(ed),
                                                   int(capacity), reps), allow=(DS_ECAPACITY, DS_ENOTCONV))
        return phi, list(M), list(off), es, ed, list(reps), rc

    # -- stage-wise --------------------------------------------------------------
    def extract(self, target, options=None):
        opts = options or Options()
        cg = C.c_void_p()
        self._sync_inputs()
        self._check(self.lib.ds_extract(self.h, int(target), C.byref(opts), C.byref(cg)))
        return cg

    def cgraph_info(self, cg):
        info = CGraphInfo()
        self._check(self.lib.ds_cgraph_get_info(cg, C.byref(info)))
        return info

    def cgraph_edges(self, cg):
        t = self.torch
        n = self.cgraph_info(cg).num_players
        es = t.empty(max(n, 1), dtype=t.int64, device=self.device)
        ed = t.empty(max(n, 1), dtype=t.int64, device=self.device)
        self._check(self.lib.ds_cgraph_edges(self.h, cg, _ptr(es), _ptr(ed)))
        return es[:n], ed[:n]

    def cgraph_nodes(self, cg):
        t = self.torch
        V = self.cgraph_info(cg).num_nodes
        gid = t.empty(V, dtype=t.int64, device=self.device)
        hop = t.empty(V, dtype=t.int32, device=self.device)
        self._check(self.lib.ds_cgraph_nodes(self.h, cg, _ptr(gid), _ptr(hop)))
        return gid, hop

    def cgraph_first_transform(self, cg):
        t = self.torch
        V = self.cgraph_info(cg).num_nodes
        out = t.empty((V, self.first_width), dtype=t.float32, device=self.device)
        self._check(self.lib.ds_cgraph_first_transform(self.h, cg, _ptr(out)))
        return out

    def cgraph_free(self, cg):
        self._check(self.lib.ds_cgraph_free(self.h, cg))

    def sample(self, n, n_samples, seed, tag, options=None):
        """ds_sample, or ds_sample_ex when `options` is given."""
        t = self.torch
        k, _ = sample_plan(n, n_samples)
        W = (n + 63) // 64
        Z = t.empty((max(k, 1), max(W, 1)), dtype=t.int64, device=self.device)
        w = t.empty(max(k, 1), dtype=t.float32, device=self.device)
        sz = t.empty(max(k, 1), dtype=t.int32, device=self.device)
        kout = C.c_int64()
        if options is None:
            self._check(self.lib.ds_sample(self.h, int(n), int(n_samples), C.c_uint64(int(seed)),
                                           C.c_uint32(int(tag) & 0xFFFFFFFF), _ptr(Z), _ptr(w), _ptr(sz),
                                           C.byref(kout)))
        else:
            self._check(self.lib.ds_sample_ex(self.h, int(n), int(n_samples), C.c_uint64(int(seed)),
                                              C.c_uint32(int(tag) & 0xFFFFFFFF), C.byref(options), _ptr(Z), _ptr(w),
                                              _ptr(sz), C.byref(kout)))
        assert kout.value == k
        return Z[:k], w[:k], sz[:k]

    def sample_range(self, n, n_samples, seed, tag, pair_begin, pair_end):
        t = self.torch
        rows = 2 * (pair_end - pair_begin)
        W = (n + 63) // 64
        Z = t.empty((max(rows, 1), max(W, 1)), dtype=t.int64, device=self.device)
        w = t.empty(max(rows, 1), dtype=t.float32, device=self.device)
        sz = t.empty(max(rows, 1), dtype=t.int32, device=self.device)
        self._check(self.lib.ds_sample_range(self.h, int(n), int(n_samples), C.c_uint64(int(seed)),
                                             C.c_uint32(int(tag) & 0xFFFFFFFF), int(pair_begin),
                                             int(pair_end), _ptr(Z), _ptr(w), _ptr(sz)))
        return Z[:rows], w[:rows], sz[:rows]

    def eval(self, cg, Z, score=DS_SCORE_PROB, pairs=False):
        """ds_eval, or ds_eval_pairs when `pairs` (rows 2r, 2r+1 complementary)."""
        t = self.torch
        Z = Z.contiguous()
        k = Z.shape[0]
        y = t.empty(max(k, 1), dtype=t.float32, device=self.device)
        pc = C.c_int32()
        self._sync_inputs()
        fn = self.lib.ds_eval_pairs if pairs else self.lib.ds_eval
        self._check(fn(self.h, cg, _ptr(Z), k, score, _ptr(y), C.byref(pc)))
        return y[:k], pc.value

    def eval_noalloc(self, cg, Z, y, score=DS_SCORE_PROB):
        """ds_eval_noalloc into the caller's y (float32[k]); queued on the context's stream, no synchronisation."""
        self._sync_inputs()
        self._check(self.lib.ds_eval_noalloc(self.h, cg, _ptr(Z), Z.shape[0], score, _ptr(y)))

    def synchronize(self):
        """Wait for the library's stream (the one given at creation, else the default stream)."""
        if self._stream is not None:
            self._stream.synchronize()
        else:
            self.torch.cuda.synchronize(self.device)

    def fidelity(self, cg, phi, ks, score=DS_SCORE_PROB, want_masks=False):
        """(fid_plus, fid_minus[, masks]) for the top-k sub-graphs, k in ks."""
        t = self.torch
        T = len(ks)
        n = self.cgraph_info(cg).num_players
        phi = phi.contiguous()
        kk = (C.c_int64 * T)(*[int(x) for x in ks])
        fp, fm = (C.c_float * T)(), (C.c_float * T)()
        masks = t.empty((2 * T, max((n + 63) // 64, 1)), dtype=t.int64, device=self.device) if want_masks else None
        self._sync_inputs()
        self._check(self.lib.ds_fidelity(self.h, cg, _ptr(phi), kk, T, score, fp, fm, _ptr(masks)))
        out = (list(fp), list(fm))
        return out + (masks,) if want_masks else out

    def copy_probe(self, nbytes):
        """Plain device copy of nbytes (calibration of profiler byte counters)."""
        t = self.torch
        src = t.zeros(nbytes // 8, dtype=t.int64, device=self.device)
        dst = t.empty_like(src)
        self._sync_inputs()
        self._check(self.lib.ds_copy_probe(self.h, _ptr(dst), _ptr(src), int(nbytes)))

    def solve(self, n, Z, w, y, options=None, allow_not_converged=False):
        t = self.torch
        opts = options or Options()
        Z, w, y = Z.contiguous(), w.contiguous(), y.contiguous()
        phi = t.empty(n, dtype=t.float32, device=self.device)
        rep = Report()
        self._sync_inputs()
        rc = self._check(self.lib.ds_solve(self.h, int(n), Z.shape[0], _ptr(Z), _ptr(w), _ptr(y),
                                           C.byref(opts), _ptr(phi), C.byref(rep)),
                         allow=(DS_ENOTCONV,) if allow_not_converged else ())
        return phi, rep, rc
