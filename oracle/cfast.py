"""ctypes access to oracle.c (the plain-C restatement of the oracle for large inputs).

TEST INFRASTRUCTURE ONLY. `build()` compiles oracle.c with gcc; nothing here touches
the HIP library.
"""
import ctypes as C
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle.c")
LIB = os.path.join(HERE, "liboracle_c.so")
_lib = None


def build(force=False):
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC",
                        "-o", LIB, SRC, "-lm"], check=True)
    return LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(LIB)
        L.oc_plan.restype = C.c_int64
        L.oc_normal_residual.restype = C.c_double
        _lib = L
    return _lib


def threads():
    """OpenMP threads the C oracle's parallel loops run on."""
    return int(lib().oc_threads())


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def philox(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oc_philox4x32_10(_p(c), _p(k), _p(out))
    return tuple(int(x) for x in out)


def plan(n, n_samples):
    H = n // 2
    b = np.zeros(H + 1, dtype=np.int64)
    wtab = np.zeros(H + 1, dtype=np.float32)
    en = C.c_int32()
    k = lib().oc_plan(C.c_int64(n), C.c_int64(n_samples), _p(b), _p(wtab), C.byref(en))
    return int(k), bool(en.value), b, wtab


def sample(n, n_samples, seed, tag, pair_range=None):
    k, en, b, wtab = plan(n, n_samples)
    r0, r1 = (0, k // 2) if pair_range is None else pair_range
    rows, W = 2 * (r1 - r0), (n + 63) // 64
    Z = np.zeros((rows, W), dtype=np.uint64)
    w = np.zeros(rows, dtype=np.float32)
    sz = np.zeros(rows, dtype=np.int32)
    lib().oc_sample_pairs(C.c_int64(n), C.c_int64(n_samples), C.c_uint64(seed), C.c_uint32(tag & 0xFFFFFFFF),
                          C.c_int64(r0), C.c_int64(r1), _p(Z), _p(w), _p(sz))
    return Z, w, sz


def gcn_values(cg, X_global, weights, Z, biases=None, score="prob", pred_class=None, bf16=False):
    """y (and the logits) of the coalitions in Z (uint64[rows, W]) on computational graph `cg`
    (as returned by oracle.compgraph.extract)."""
    V, n = cg["num_nodes"], cg["num_players"]
    Xc = np.ascontiguousarray(np.asarray(X_global, dtype=np.float64)[cg["node_gid"]])
    dims = np.array([weights[0].shape[0]] + [w.shape[1] for w in weights], dtype=np.int32)
    Wcat = np.concatenate([np.asarray(w, dtype=np.float64).ravel() for w in weights])
    bcat = None
    if biases is not None:
        bcat = np.concatenate([np.zeros(dims[l + 1]) if b is None else np.asarray(b, dtype=np.float64)
                               for l, b in enumerate(biases)])
    psrc = np.ascontiguousarray(cg["lsrc"], dtype=np.int32)
    pdst = np.ascontiguousarray(cg["ldst"], dtype=np.int32)
    Z = np.ascontiguousarray(Z, dtype=np.uint64)
    rows = Z.shape[0]
    C_ = int(dims[-1])
    if pred_class is None:
        full = np.zeros((1, (n + 63) // 64), dtype=np.uint64)
        bits = np.ones((1, n), dtype=bool)
        from .sampling import pack_rows
        full = pack_rows(bits) if n else full
        y1 = np.zeros(1)
        lg = np.zeros((1, C_))
        lib().oc_gcn_values(C.c_int32(V), C.c_int64(n), _p(psrc), _p(pdst), C.c_int32(0 if cg["undirected"] else 1),
                            _p(Xc), C.c_int32(len(weights)), _p(dims), _p(Wcat), _p(bcat) if bcat is not None else None,
                            C.c_int32(int(bf16)), C.c_int32(1), C.c_int32(0), _p(full), C.c_int64(1), _p(y1), _p(lg))
        pred_class = int(np.argmax(lg[0]))
    y = np.zeros(rows)
    logits = np.zeros((rows, C_))
    lib().oc_gcn_values(C.c_int32(V), C.c_int64(n), _p(psrc), _p(pdst), C.c_int32(0 if cg["undirected"] else 1),
                        _p(Xc), C.c_int32(len(weights)), _p(dims), _p(Wcat), _p(bcat) if bcat is not None else None,
                        C.c_int32(int(bf16)), C.c_int32(1 if score == "logit" else 0), C.c_int32(pred_class),
                        _p(Z), C.c_int64(rows), _p(y), _p(logits))
    return y, pred_class, logits


def cgls(n, Z, w, y, tol=1e-10, max_iter=None):
    Z = np.ascontiguousarray(Z, dtype=np.uint64)
    w = np.ascontiguousarray(w, dtype=np.float32)
    y = np.ascontiguousarray(y, dtype=np.float64)
    if max_iter is None:
        max_iter = min(max(n, 1), 10000)
    phi = np.zeros(n)
    it, rel = C.c_int64(), C.c_double()
    lib().oc_cgls(C.c_int64(n), C.c_int64(Z.shape[0]), _p(Z), _p(w), _p(y), C.c_double(tol), C.c_int64(max_iter),
                  _p(phi), C.byref(it), C.byref(rel))
    return phi, it.value, rel.value


def normal_residual(n, Z, w, y, phi):
    Z = np.ascontiguousarray(Z, dtype=np.uint64)
    w = np.ascontiguousarray(w, dtype=np.float32)
    y = np.ascontiguousarray(y, dtype=np.float64)
    phi = np.ascontiguousarray(phi, dtype=np.float64)
    return float(lib().oc_normal_residual(C.c_int64(n), C.c_int64(Z.shape[0]), _p(Z), _p(w), _p(y), _p(phi)))
