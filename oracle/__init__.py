"""CPU oracle of the DASGD/SGNS worker step -- TEST INFRASTRUCTURE ONLY.

``tensair_oracle.c`` is the plain sequential statement of the step (double
arithmetic); this module builds it with gcc and wraps it with ctypes/numpy.
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import it.  Nothing under ``oracle/`` imports the product package;
``oracle/driver.py`` takes its seeded inputs from ``workload.py`` at the repository
root, which holds none of the method's arithmetic and belongs to neither side.

Paper: TensAIR, arXiv 2211.10280 -- Eq. 1, Algorithm 1 (train), Section 3.1
(staleness and ordering), Section 4 (sparse updates).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tensair_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, BF16, F64 = 0, 1, 2
_NP = {F32: np.float32, BF16: np.uint16, F64: np.float64}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add contraction, so the
    single-precision initialisation is evaluated exactly as written)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_SAN_SRC = os.path.join(_HERE, "sanitize_check.c")
_SAN_BIN = os.path.join(_HERE, "sanitize_check")


def build_sanitize_check(force: bool = False) -> str:
    """Compile ``sanitize_check.c`` (the oracle's C source driven over small inputs) with gcc's address and
    undefined-behaviour sanitizers into a program of its own; the CPU tests run it."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SAN_SRC))
    if force or not os.path.exists(_SAN_BIN) or os.path.getmtime(_SAN_BIN) < newest:
        subprocess.check_call(
            ["gcc", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-fsanitize=address,undefined",
             "-static-libasan", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
             "-o", _SAN_BIN, _SAN_SRC, "-lm"])
    return _SAN_BIN


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, i32, i64, u32, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64
        L.orc_philox4x32_10.argtypes = [vp, vp, vp]
        L.orc_philox4x32_10.restype = None
        L.orc_alias_build.argtypes = [vp, i64, vp, vp]
        L.orc_alias_build.restype = C.c_int
        L.orc_pairs.argtypes = [i64, i32, i64, i32, vp, vp]
        L.orc_pairs.restype = i64
        L.orc_sample_negatives.argtypes = [i64, vp, vp, u64, u32, u32, i64, vp, vp, i32, vp]
        L.orc_sample_negatives.restype = None
        L.orc_sample_negatives_resampled.argtypes = [i64, vp, vp, u64, u32, u32, i64, vp, vp, i32, vp, i32, vp]
        L.orc_sample_negatives_resampled.restype = None
        L.orc_init_tables.argtypes = [i64, i32, i32, C.c_int, u64, vp, vp]
        L.orc_init_tables.restype = None
        L.orc_sgns_grad.argtypes = [vp, i64, i32, i32, i64, i32, i64, i32, i32, C.c_int,
                                    vp, vp, vp, vp, u64, u32, u32, vp]
        L.orc_sgns_grad.restype = vp
        L.orc_grad_sizes.argtypes = [vp, vp, vp, vp]
        L.orc_grad_sizes.restype = None
        L.orc_grad_loss.argtypes = [vp]
        L.orc_grad_loss.restype = C.c_double
        L.orc_grad_export.argtypes = [vp] * 10
        L.orc_grad_export.restype = None
        L.orc_grad_free.argtypes = [vp]
        L.orc_grad_free.restype = None
        L.orc_dasgd_apply_table.argtypes = [i64, i32, i32, C.c_int, vp, i32, vp, vp, vp, C.c_float]
        L.orc_dasgd_apply_table.restype = None
        L.orc_dasgd_apply_table_sr.argtypes = [i64, i32, i32, C.c_int, vp, i32, vp, vp, vp, C.c_float, u64, u32, u32]
        L.orc_dasgd_apply_table_sr.restype = None
        L.orc_double_to_bf16.argtypes = [C.c_double]
        L.orc_double_to_bf16.restype = C.c_uint16
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ---------------------------------------------------------------- primitives
def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def alias_build(counts):
    counts = np.ascontiguousarray(counts, dtype=np.uint64)
    V = counts.shape[0]
    thr = np.zeros(V, dtype=np.uint32)
    alias = np.zeros(V, dtype=np.int32)
    rc = lib().orc_alias_build(_p(counts), V, _p(thr), _p(alias))
    if rc != 0:
        raise ValueError("alias_build: no id has a positive count")
    return thr, alias


def pairs(T, w, begin, n):
    P = lib().orc_pairs(T, w, begin, n, None, None)
    pos = np.zeros(max(P, 1), dtype=np.int64)
    q = np.zeros(max(P, 1), dtype=np.int32)
    lib().orc_pairs(T, w, begin, n, _p(pos), _p(q))
    return pos[:P], q[:P]


def sample_negatives(V, thr, alias, seed, worker, epoch, pos, q, N, resample_tok=None, w=None):
    """The N negatives of every pair (pos, q).  With ``resample_tok`` (the token stream) and the window
    ``w``: the variant in which a negative equal to the pair's center or context word is drawn once
    more, from the other two words of the same Philox block."""
    pos = np.ascontiguousarray(pos, dtype=np.int64)
    q = np.ascontiguousarray(q, dtype=np.int32)
    P = pos.shape[0]
    out = np.zeros((P, N), dtype=np.int32)
    if resample_tok is None:
        lib().orc_sample_negatives(V, _p(thr), _p(alias), seed, worker, epoch, P, _p(pos), _p(q), N, _p(out))
    else:
        tok = np.ascontiguousarray(resample_tok, dtype=np.int32)
        lib().orc_sample_negatives_resampled(V, _p(thr), _p(alias), seed, worker, epoch, P, _p(pos), _p(q), N,
                                             _p(tok), w, _p(out))
    return out


def double_to_bf16(x: float) -> int:
    return int(lib().orc_double_to_bf16(float(x)))


def bf16_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32)


def init_tables(V, D, stride, dtype, seed):
    w_in = np.zeros((V, stride), dtype=_NP[dtype])
    w_out = np.zeros((V, stride), dtype=_NP[dtype])
    lib().orc_init_tables(V, D, stride, dtype, seed, _p(w_in), _p(w_out))
    return w_in, w_out


# ---------------------------------------------------------------- gradient
@dataclass
class SparseRows:
    ids: np.ndarray      # int32 [U] ascending unique
    rows: np.ndarray     # float32 [U, D]
    seg: np.ndarray      # int64 [U+1] occurrence offsets
    rows64: np.ndarray | None = None


@dataclass
class Grad:
    P: int
    loss: float
    negatives: np.ndarray   # int32 [P, N]
    gin: SparseRows
    gout: SparseRows


def sgns_grad(tok, w, N, begin, n_centers, D, dtype, W_in, W_out, thr, alias,
              seed, worker, epoch, neg_override=None, want64=False, resample=False) -> Grad:
    """calculate_gradient of Algorithm 1 for one mini-batch of centers.  ``resample``: the variant
    of ``sample_negatives`` that draws colliding negatives once more."""
    tok = np.ascontiguousarray(tok, dtype=np.int32)
    T = tok.shape[0]
    V, stride = W_in.shape
    if resample and neg_override is None:
        pos, q = pairs(T, w, begin, n_centers)
        neg_override = sample_negatives(V, thr, alias, seed, worker, epoch, pos, q, N, resample_tok=tok, w=w)
    assert W_in.dtype == _NP[dtype] and W_out.dtype == _NP[dtype]
    assert W_in.flags.c_contiguous and W_out.flags.c_contiguous
    if neg_override is not None:
        neg_override = np.ascontiguousarray(neg_override, dtype=np.int32)
    L = lib()
    h = L.orc_sgns_grad(_p(tok), T, w, N, begin, n_centers, V, D, stride, dtype,
                        _p(W_in), _p(W_out), _p(thr), _p(alias), seed, worker, epoch,
                        _p(neg_override))
    try:
        P, Ui, Uo = C.c_int64(), C.c_int64(), C.c_int64()
        L.orc_grad_sizes(h, C.byref(P), C.byref(Ui), C.byref(Uo))
        P, Ui, Uo = P.value, Ui.value, Uo.value
        gi = SparseRows(np.zeros(Ui, np.int32), np.zeros((Ui, D), np.float32), np.zeros(Ui + 1, np.int64),
                        np.zeros((Ui, D), np.float64) if want64 else None)
        go = SparseRows(np.zeros(Uo, np.int32), np.zeros((Uo, D), np.float32), np.zeros(Uo + 1, np.int64),
                        np.zeros((Uo, D), np.float64) if want64 else None)
        neg = np.zeros((P, N), dtype=np.int32)
        L.orc_grad_export(h, _p(gi.ids), _p(gi.rows), _p(gi.rows64), _p(gi.seg),
                          _p(go.ids), _p(go.rows), _p(go.rows64), _p(go.seg), _p(neg))
        loss = L.orc_grad_loss(h)
    finally:
        L.orc_grad_free(h)
    return Grad(P, loss, neg, gi, go)


# ---------------------------------------------------------------- apply
def dasgd_apply_table(W, D, dtype, sources, lr, stochastic=None):
    """apply_gradient of Algorithm 1 / Eq. 1 on one table, in place.
    ``sources`` = list of (ids int32[U_k], rows float32[U_k, D]); source 0 is the own
    gradient, the others are peers' (same alpha, summed).
    ``stochastic`` = (seed, serial, table): the variant in which a bfloat16 table is rounded
    stochastically (see ``stochastic_bf16`` in the C source); ignored for float tables."""
    V, stride = W.shape
    assert W.dtype == _NP[dtype] and W.flags.c_contiguous
    K = len(sources)
    ids = [np.ascontiguousarray(s[0], dtype=np.int32) for s in sources]
    rows = [np.ascontiguousarray(s[1], dtype=np.float32) for s in sources]
    n = np.array([i.shape[0] for i in ids], dtype=np.int64)
    idp = (C.c_void_p * max(K, 1))(*[i.ctypes.data for i in ids])
    rwp = (C.c_void_p * max(K, 1))(*[r.ctypes.data for r in rows])
    if stochastic is None:
        lib().orc_dasgd_apply_table(V, D, stride, dtype, _p(W), K, _p(n), idp, rwp, np.float32(lr))
    else:
        seed, serial, table = stochastic
        lib().orc_dasgd_apply_table_sr(V, D, stride, dtype, _p(W), K, _p(n), idp, rwp, np.float32(lr),
                                       seed, serial, table)


def dasgd_apply(W_in, W_out, D, dtype, grads, lr, stochastic=None):
    """Merged application of the own gradient grads[0] and peer gradients grads[1:].
    ``stochastic`` = (seed, serial): stochastic rounding of bfloat16 tables (a variant)."""
    sr = (lambda t: None) if stochastic is None else (lambda t: (stochastic[0], stochastic[1], t))
    dasgd_apply_table(W_in, D, dtype, [(g.gin.ids, g.gin.rows) for g in grads], lr, sr(0))
    dasgd_apply_table(W_out, D, dtype, [(g.gout.ids, g.gout.rows) for g in grads], lr, sr(1))


# ---------------------------------------------------------------- gradient buffer
def grad_add_rows(a, b, D):
    """``gradients += gradient`` of Algorithm 1 (train) for one table's sparse rows.

    The buffer of gradients that have not been sent yet and a new gradient are both lists
    of (ascending unique row ids, rows); their sum lists the union of the ids, a row that
    only one of them has is taken over, a row that both have is added.  The buffer lives
    in the boundary's format, float32, so every ``+=`` rounds once: the sum is taken in
    double and rounded to float (which is the correctly rounded float sum).  A listed row
    stays listed even if it sums to zero.  a, b: (ids int32[U], rows float32[U, D])."""
    ia, ra = np.asarray(a[0], dtype=np.int32), np.asarray(a[1], dtype=np.float32).reshape(-1, D)
    ib, rb = np.asarray(b[0], dtype=np.int32), np.asarray(b[1], dtype=np.float32).reshape(-1, D)
    ids = np.union1d(ia, ib).astype(np.int32)
    acc = np.zeros((ids.shape[0], D), dtype=np.float64)
    acc[np.searchsorted(ids, ia)] += ra.astype(np.float64)
    acc[np.searchsorted(ids, ib)] += rb.astype(np.float64)
    return ids, acc.astype(np.float32)


def grad_add(a: Grad, b: Grad, D: int) -> Grad:
    """Sum of two sparse gradients, table by table (segment offsets and negatives do not
    apply to a sum and are left empty)."""
    gi = grad_add_rows((a.gin.ids, a.gin.rows), (b.gin.ids, b.gin.rows), D)
    go = grad_add_rows((a.gout.ids, a.gout.rows), (b.gout.ids, b.gout.rows), D)
    none = np.zeros(0, np.int64)
    return Grad(a.P + b.P, float("nan"), np.zeros((0, 0), np.int32),
                SparseRows(gi[0], gi[1], none), SparseRows(go[0], go[1], none))


# ---------------------------------------------------------------- gradient messages in bfloat16
def grad_pack_rows(rows):
    """A gradient message whose rows travel as bfloat16 -- a variant beyond the paper, which sends
    float gradients and names gradient application and the network as what limits Word2Vec
    scaling (Section 4.3).  Every element of the float32 rows is rounded to the nearest
    bfloat16, ties to even: the candidates are the bfloat16 values at and above |x| (the float's
    upper 16 bits, and that plus one unit in the last place), the nearer one is taken, measured
    in double; beyond the largest finite bfloat16 the upper candidate counts as 2^128, so that
    what lies past the midpoint becomes infinity; infinities keep their sign, NaN becomes
    0x7FC0.  rows: float32 array; returns uint16 bits of the same shape."""
    x = np.ascontiguousarray(rows, dtype=np.float32)
    bits = x.view(np.uint32)
    sign = (bits >> np.uint32(31)).astype(np.uint16) << np.uint16(15)
    mag = np.abs(x.astype(np.float64))
    lo = (bits & np.uint32(0x7FFF0000)).astype(np.uint32)      # magnitude truncated to bfloat16
    hi = (lo + np.uint32(0x10000)).astype(np.uint32)
    lo_v = lo.view(np.float32).astype(np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        hi_v = np.where(hi >= np.uint32(0x7F800000), 2.0 ** 128, hi.view(np.float32).astype(np.float64))
        d_lo, d_hi = mag - lo_v, hi_v - mag
    odd = ((lo >> np.uint32(16)) & np.uint32(1)) == 1
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & odd)
    out = (np.where(take_hi, hi, lo) >> np.uint32(16)).astype(np.uint16) | sign
    out = np.where(np.isinf(x), np.uint16(0x7F80) | sign, out)
    out = np.where(np.isnan(x), np.uint16(0x7FC0), out)
    return out.astype(np.uint16)


def grad_unpack_rows(bits):
    """The float32 rows a receiver sees in a bfloat16 gradient message (exact widening)."""
    return bf16_to_f32(np.asarray(bits, dtype=np.uint16))


def grad_through_bf16(g: Grad) -> Grad:
    """A gradient as its receiver sees it after travelling as a bfloat16 message: same rows
    listed, every element rounded once."""
    r = lambda s: SparseRows(s.ids, grad_unpack_rows(grad_pack_rows(s.rows)), s.seg)
    return Grad(g.P, g.loss, g.negatives, r(g.gin), r(g.gout))


# ---------------------------------------------------------------- dense model, predict path, drift metric
def dense_apply(theta, dtype, grads, lr):
    """apply_gradient of Algorithm 1 / Eq. 1 for a dense model (Section 4, "Sparse vs. Dense
    Models": every variable receives gradient), in place: theta <- theta - alpha * sum_k g_k
    for the own gradient and the gradients received from peers, summed in double, one rounded
    store per element.  theta: 1-D array in its own type (float32, or uint16 bfloat16 bits);
    grads: list of float32 arrays of the same length; alpha enters as (double)(float)lr."""
    assert theta.ndim == 1 and theta.dtype == _NP[dtype]
    acc = np.zeros(theta.shape[0], dtype=np.float64)
    for g in grads:
        g = np.asarray(g, dtype=np.float32)
        assert g.shape == theta.shape
        acc += g.astype(np.float64)
    alpha = float(np.float32(lr))
    if dtype == BF16:
        new = bf16_to_f32(theta).astype(np.float64) - alpha * acc
        theta[:] = _bf16_round(new)
    else:
        theta[:] = (theta.astype(np.float64) - alpha * acc).astype(theta.dtype)
    return theta


def _bf16_round(x64: np.ndarray) -> np.ndarray:
    """double -> bfloat16 bits, round to nearest even, vectorised (finite inputs).
    The candidate below x is found from the float32 truncation, then the nearer of the two
    neighbouring bfloat16 values is taken in double, ties to the even one."""
    f = x64.astype(np.float32)                       # may already round up; fix below in double
    bits = f.view(np.uint32)
    lo = (bits & np.uint32(0xFFFF0000))
    lo_v = lo.view(np.float32).astype(np.float64)
    # make lo the bfloat16 value at or below |x| (towards zero)
    toward = np.abs(lo_v) > np.abs(x64)
    lo = np.where(toward, lo - np.uint32(0x10000), lo).astype(np.uint32)
    lo_v = lo.view(np.float32).astype(np.float64)
    hi = (lo + np.uint32(0x10000)).astype(np.uint32)
    hi_v = hi.view(np.float32).astype(np.float64)
    d_lo, d_hi = np.abs(x64 - lo_v), np.abs(hi_v - x64)
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (((lo >> np.uint32(16)) & np.uint32(1)) == 1))
    return (np.where(take_hi, hi, lo) >> np.uint32(16)).astype(np.uint16)


def lookup(W, dtype, D, ids):
    """predict of Algorithm 1 for an embedding model: the vectors of the given words (rows of
    the table, widened to float32; padding columns dropped)."""
    ids = np.asarray(ids, dtype=np.int64)
    rows = W[ids, :D]
    return bf16_to_f32(rows) if dtype == BF16 else rows.astype(np.float32)


def cosine_difference(A, B, dtype, D):
    """Section 4.4: difference between the embeddings of every word before (A) and after (B)
    further training, 1 - cos(A[r], B[r]) per row, in double.  Where the paper is silent: a
    row that is zero in both tables has difference 0, one that is zero in only one has 1."""
    a = (bf16_to_f32(A[:, :D]) if dtype == BF16 else A[:, :D]).astype(np.float64)
    b = (bf16_to_f32(B[:, :D]) if dtype == BF16 else B[:, :D]).astype(np.float64)
    dot = (a * b).sum(axis=1)
    na, nb = (a * a).sum(axis=1), (b * b).sum(axis=1)
    out = np.ones(a.shape[0], dtype=np.float64)
    ok = (na > 0) & (nb > 0)
    out[ok] = 1.0 - dot[ok] / np.sqrt(na[ok] * nb[ok])
    out[(na == 0) & (nb == 0)] = 0.0
    return out


# ---------------------------------------------------------------- staleness
def staleness(G_i, G_j) -> int:
    """Section 3.1: |G_i u G_j| - |G_i n G_j| for the set G_i of gradients model i had
    applied when it computed a gradient and the set G_j model j has applied when it
    applies that gradient."""
    G_i, G_j = set(G_i), set(G_j)
    return len(G_i | G_j) - len(G_i & G_j)
