"""Coalition sampling plan: size-stratified allocation, complementary pairs,
exact-size random masks, and per-row kernel weights.

Follows the paper's sampling section: the number of samples of each coalition
size is proportional to the total Shapley-kernel mass of that size (the
sample-distribution equation), every sampled coalition comes with its
complement, and pairs are laid out sorted by size.  Points the paper leaves
open (rounding, how a row of a given size is drawn, the per-row weight) are
fixed here as follows:

* k = 2*floor(n_samples/2) rows.  Pair 0 is (empty, full).  K = k/2 - 1
  sampled pairs.  If n <= 24 and n_samples >= 2^n every coalition is
  enumerated instead (k = 2^n; pair r = (bit pattern r, its complement)).
* pair classes s = 1..H, H = floor(n/2): a pair of sizes (s, n-s).  Class mass
  pi_s = rho_s (if 2s == n) else 2*rho_s, rho_s = (n-1)/(s*(n-s)).  With
  c_s the running sum of pi and T = c_H, the class boundaries are
  b_s = floor(K*(c_s/T) + 0.5) (b_H = K), and pair r in [1, K] has the small
  size s(r) = min{s : b_s >= r}.
* row 2r of pair r = the s(r) columns with the smallest (key, column) where
  key(r, j) is word j%4 of Philox4x32-10 with key (seed_lo, seed_hi) and
  counter (j//4, r_lo, r_hi, tag); row 2r+1 is its complement.
* a row of size s weighs rho_s / m_s with m_s the number of emitted rows of
  that size (so each represented size class carries exactly its kernel mass;
  under enumeration m_s = C(n, s) and the weight is the Shapley kernel itself).
* option saturate=True (a refinement, off by default): a size class that is allotted at least
  as many pairs as it has coalitions, q_s >= C(n, s), is enumerated instead of sampled: its
  C(n, s) pairs are the s-subsets of the players in lexicographic order, each once, with the
  Shapley kernel weight itself, rho_s / C(n, s). The pairs this frees are allotted to the
  other classes by the same rule (cumulative rounding over the classes that are left), and the
  test is repeated for the next class. C(n, s) grows and the allotment shrinks with s, so
  the enumerated classes are s = 1..S_e. The class 2s = n is never enumerated this way.
"""
from math import comb
import numpy as np

from .philox import philox4x32_10_array

ENUM_MAX_PLAYERS = 24


def row_count(n, n_samples):
    """(k, enumerate?)"""
    if n <= ENUM_MAX_PLAYERS and n_samples >= (1 << n):
        return 1 << n, True
    return 2 * (int(n_samples) // 2), False


def rho(n, s):
    """Total kernel mass of all coalitions of size s (sample-distribution eq.)."""
    return float(n - 1) / (float(s) * float(n - s))


def allocation(n, n_samples, weighting="class", saturate=False):
    """Class boundaries b[0..H], pairs per class q[1..H], weight table
    wtab[1..H] (float32; entry 0 unused and zero).

    weighting="class" (default): a row of size s weighs rho_s / (rows of that size).
    weighting="uniform": every sampled row weighs 1 -- the rows are already allocated in
    proportion to rho_s, so this is the importance-sampling form of the same estimator (it
    differs from the default only through the rounding of the allocation and through classes
    that received no row).  Enumerated plans keep the exact kernel weights."""
    if weighting not in ("class", "uniform"):
        raise ValueError("weighting must be 'class' or 'uniform'")
    if saturate and weighting != "class":
        raise ValueError("saturate needs the class-mass weighting")
    k, enum = row_count(n, n_samples)
    H = n // 2
    out = {"n": n, "k": k, "enumerate": enum, "H": H}
    if enum:
        wtab = np.zeros(H + 1, dtype=np.float32)
        for s in range(1, H + 1):
            wtab[s] = np.float32(rho(n, s) / float(comb(n, s)))
        out.update(K=k // 2 - 1, b=None, q=None, wtab=wtab)
        return out
    K = k // 2 - 1
    enum_upto, used = 0, 0                    # classes 1..enum_upto are enumerated and take `used` pairs
    while True:
        # the K - used pairs that are left, over the classes enum_upto+1..H
        c = np.zeros(H + 1, dtype=np.float64)
        acc = 0.0
        for s in range(enum_upto + 1, H + 1):
            r = rho(n, s)
            acc = acc + (r if 2 * s == n else 2.0 * r)
            c[s] = acc
        T = acc
        b = np.zeros(H + 1, dtype=np.int64)
        for s in range(1, enum_upto + 1):
            b[s] = b[s - 1] + comb(n, s)
        for s in range(enum_upto + 1, H):
            b[s] = used + int(np.floor(float(K - used) * (c[s] / T) + 0.5))
        if H >= 1:
            b[H] = K
        s1 = enum_upto + 1
        if not saturate or s1 > H or 2 * s1 >= n:
            break
        cap = comb(n, s1)
        if int(b[s1]) - used >= cap:          # (then used + cap <= b[s1] <= K)
            enum_upto, used = s1, used + cap
            continue
        break
    q = np.diff(b, prepend=0)
    q[0] = 0
    wtab = np.zeros(H + 1, dtype=np.float32)
    for s in range(1, H + 1):
        m = int(q[s]) * (2 if 2 * s == n else 1)
        if m > 0:
            wtab[s] = np.float32(1.0) if weighting == "uniform" else np.float32(rho(n, s) / float(m))
    out.update(K=K, b=b, q=q, wtab=wtab, T=T, enum_upto=enum_upto)
    return out


def unrank_subset(n, s, j):
    """The j-th (from 0) s-subset of {0..n-1} in lexicographic order, as an ascending list: element x
    is the next one if fewer than C(n-1-x, remaining-1) subsets start with it ... else skip those."""
    out, x = [], 0
    for i in range(s):
        while True:
            c = comb(n - 1 - x, s - 1 - i)    # subsets that continue with element x
            if j < c:
                break
            j -= c
            x += 1
        out.append(x)
        x += 1
    return out


def pair_sizes(b, r):
    """Small-member size of pairs r (array of pair indices in [1, K])."""
    return np.searchsorted(b, np.asarray(r), side="left")


def keys_for_pairs(n, pairs, seed, tag):
    """Philox keys kappa(r, j) for the given pair indices: uint64[len(pairs), n]."""
    pairs = np.asarray(pairs, dtype=np.uint64)
    nq = (n + 3) // 4
    c0 = np.arange(nq, dtype=np.uint64)[None, :]
    c1 = (pairs & np.uint64(0xFFFFFFFF))[:, None]
    c2 = (pairs >> np.uint64(32))[:, None]
    c3 = np.uint64(int(tag) & 0xFFFFFFFF)
    o = philox4x32_10_array(c0, c1, c2, c3, int(seed) & 0xFFFFFFFF,
                            (int(seed) >> 32) & 0xFFFFFFFF)
    keys = np.stack(np.broadcast_arrays(*o), axis=-1).reshape(len(pairs), nq * 4)
    return keys[:, :n]


def pack_rows(bits):
    """bool[rows, n] -> uint64[rows, ceil(n/64)], column j -> word j>>6, bit j&63."""
    rows, n = bits.shape
    W = (n + 63) // 64
    padded = np.zeros((rows, W * 64), dtype=np.uint8)
    padded[:, :n] = bits
    by = np.packbits(padded, axis=1, bitorder="little")
    return np.ascontiguousarray(by).view("<u8").reshape(rows, W)


def unpack_rows(Z, n):
    """uint64[rows, W] -> bool[rows, n]"""
    by = np.ascontiguousarray(Z).view(np.uint8).reshape(Z.shape[0], -1)
    return np.unpackbits(by, axis=1, bitorder="little")[:, :n].astype(bool)


def sample(n, n_samples, seed, tag, pair_range=None, chunk_elems=1 << 22, weighting="class", saturate=False):
    """Mask matrix Z (uint64[k, W]), weights w (float32[k]) and sizes sz
    (int32[k]).  With pair_range=(r0, r1) only the rows of pairs r0 <= r < r1
    are produced (rows 2*r0 .. 2*r1-1), identical to those of the full run."""
    plan = allocation(n, n_samples, weighting, saturate)
    k, K, wtab = plan["k"], plan["K"], plan["wtab"]
    r0, r1 = (0, k // 2) if pair_range is None else pair_range
    npairs = r1 - r0
    bits = np.zeros((2 * npairs, n), dtype=bool)
    w = np.zeros(2 * npairs, dtype=np.float32)
    if plan["enumerate"]:
        r = np.arange(r0, r1, dtype=np.uint64)
        small = ((r[:, None] >> np.arange(n, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(bool)
        bits[0::2] = small
        bits[1::2] = ~small
        sz = bits.sum(axis=1).astype(np.int32)
        cls = np.minimum(sz, n - sz)
        w = wtab[cls]
        w[cls == 0] = 0.0
        return pack_rows(bits), w.astype(np.float32), sz
    if r0 == 0:
        bits[1, :] = True                      # pair 0 = (empty, full), weight 0
    first = max(r0, 1)
    rows_per_chunk = max(1, chunk_elems // max(n, 1))
    for a in range(first, r1, rows_per_chunk):
        pr = np.arange(a, min(r1, a + rows_per_chunk), dtype=np.int64)
        s = pair_sizes(plan["b"], pr)
        keys = keys_for_pairs(n, pr, seed, tag)
        order = np.argsort(keys, axis=1, kind="stable")    # (key, column) order
        rank = np.empty_like(order)
        np.put_along_axis(rank, order, np.arange(n)[None, :], axis=1)
        small = rank < s[:, None]
        for i in np.flatnonzero(s <= plan["enum_upto"]):   # pairs of enumerated classes: the subsets in order
            si = int(s[i])
            small[i] = False
            small[i, unrank_subset(n, si, int(pr[i]) - 1 - int(plan["b"][si - 1]))] = True
        lo = 2 * (pr - r0)
        bits[lo] = small
        bits[lo + 1] = ~small
        w[lo] = wtab[s]
        w[lo + 1] = wtab[s]
    sz = bits.sum(axis=1).astype(np.int32)
    return pack_rows(bits), w, sz
