"""ctypes front end of the CPU oracle (csgs_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg.  The product package never imports this.
All arrays are numpy; every function allocates its outputs and returns them.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csgs_oracle.c")
_LIB = os.path.join(_HERE, "libcsgs_oracle.so")

OK, EINVAL, ECAP, ERANGE, EVALUE, EEMPTY = 0, -1, -2, -3, -4, -5


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle error {code}")
        self.code = code


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared",
                               "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Stats(C.Structure):
    _fields_ = [("n_cand", C.c_int64), ("n_local", C.c_int64), ("n_remote", C.c_int64),
                ("edges_scanned", C.c_int64), ("w_local", C.c_uint64), ("w_remote", C.c_uint64),
                ("total", C.c_uint64), ("shift", C.c_int32), ("skew_fx", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_LIB)
        _lib.orc_draw_word.restype = C.c_uint64
        _lib.orc_draw_word.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32]
        _lib.orc_skew_fx.restype = C.c_int64
        _lib.orc_skew_fx.argtypes = [C.c_float]
        _lib.orc_shift.restype = C.c_int
        _lib.orc_shift.argtypes = [C.c_int32, C.c_float, C.c_float]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(rc):
    if rc != OK:
        raise OracleError(rc)


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def draw_word(seed, it, layer, t):
    return int(lib().orc_draw_word(seed, it, layer, t))


def shift_for(nS, skew, rownorm2_max=1.0):
    return int(lib().orc_shift(nS, skew, rownorm2_max))


def theorem1_skew_fx(n_cand, n_remote, B, D, s_fx_max):
    lib().orc_theorem1_skew_fx.restype = C.c_int64
    return int(lib().orc_theorem1_skew_fx(C.c_int64(n_cand), C.c_int64(n_remote), C.c_int32(B), C.c_double(D),
                                          C.c_int64(s_fx_max)))


def build_probs(g, S, skew, cap=None, auto=None):
    """g: synth.Graph-like (n_nodes,rowptr,colidx,val,local_lo,local_hi,rownorm2_max).
    skew = inf: "Local" version.  auto = (D, B): skew from Theorem 1, `skew` is then its upper bound."""
    S = np.ascontiguousarray(S, dtype=np.int32)
    cap = int(g.n_nodes if cap is None else cap)
    cand_id = np.zeros(cap, np.int32)
    cand_w = np.zeros(cap, np.uint64)
    cdf = np.zeros(cap, np.uint64)
    q = np.zeros(cap, np.float32)
    st = _Stats()
    mode = 1 if auto is not None else (2 if skew == float("inf") else 0)
    D, B = auto if auto is not None else (0.0, 0)
    rc = lib().orc_build_probs_ex(C.c_int64(g.n_nodes), _p(g.rowptr), _p(g.colidx), _p(g.val),
                                  C.c_int32(g.local_lo), C.c_int32(g.local_hi), C.c_float(g.rownorm2_max),
                                  _p(S), C.c_int32(len(S)), C.c_int(mode), C.c_float(skew), C.c_float(D), C.c_int32(B),
                                  _p(cand_id), _p(cand_w), _p(cdf), _p(q), C.c_int64(cap), C.byref(st))
    _chk(rc)
    n = st.n_cand
    return SimpleNamespace(cand_id=cand_id[:n], cand_w=cand_w[:n], cdf=cdf[:n], q=q[:n],
                           n_cand=n, n_local=st.n_local, n_remote=st.n_remote,
                           edges_scanned=st.edges_scanned, w_local=st.w_local, w_remote=st.w_remote,
                           total=st.total, shift=st.shift, skew_fx=st.skew_fx)


def _sample_common(fn_name, g, S, probs, B, tail_args, adj_cap):
    S = np.ascontiguousarray(S, dtype=np.int32)
    nS = len(S)
    if adj_cap is None:
        deg = g.rowptr[S.astype(np.int64) + 1] - g.rowptr[S.astype(np.int64)]
        adj_cap = int(deg.sum())
    S_next = np.zeros(B, np.int32)
    mult = np.zeros(B, np.int32)
    p_incl = np.zeros(B, np.float32)
    n_next = C.c_int32(0)
    adj_rowptr = np.zeros(nS + 1, np.int32)
    adj_col = np.zeros(max(adj_cap, 1), np.int32)
    adj_val = np.zeros(max(adj_cap, 1), np.float32)
    adj_nnz = C.c_int64(0)
    cand_id = np.ascontiguousarray(probs.cand_id, np.int32)
    cdf = np.ascontiguousarray(probs.cdf, np.uint64)
    rc = getattr(lib(), fn_name)(
        C.c_int64(g.n_nodes), _p(g.rowptr), _p(g.colidx), _p(g.val), _p(S), C.c_int32(nS),
        _p(cand_id), _p(cdf), C.c_int64(len(cand_id)), *tail_args,
        _p(S_next), _p(mult), _p(p_incl), C.byref(n_next),
        _p(adj_rowptr), _p(adj_col), _p(adj_val), C.c_int64(adj_cap), C.byref(adj_nnz))
    _chk(rc)
    n, nnz = n_next.value, adj_nnz.value
    return SimpleNamespace(S_next=S_next[:n], mult=mult[:n], p_incl=p_incl[:n], n_next=n,
                           adj_rowptr=adj_rowptr, adj_col=adj_col[:nnz], adj_val=adj_val[:nnz],
                           adj_nnz=nnz)


def sample_layer(g, S, probs, B, seed, it, layer, adj_cap=None):
    tail = (C.c_int32(B), C.c_uint64(seed), C.c_uint64(it), C.c_uint32(layer))
    return _sample_common("orc_sample_layer", g, S, probs, B, tail, adj_cap)


def sample_from_words(g, S, probs, words, adj_cap=None):
    words = np.ascontiguousarray(words, dtype=np.uint64)
    tail = (_p(words), C.c_int32(len(words)))
    out = _sample_common("orc_sample_from_words", g, S, probs, len(words), tail, adj_cap)
    out._words = words
    return out


def draw_nodes(probs, B, seed, it, layer):
    """Draws only (no adjacency): S_next, mult, p_incl and the inclusion probabilities in double."""
    cand_id = np.ascontiguousarray(probs.cand_id, np.int32)
    cdf = np.ascontiguousarray(probs.cdf, np.uint64)
    S_next, mult = np.zeros(B, np.int32), np.zeros(B, np.int32)
    p_incl, pd = np.zeros(B, np.float32), np.zeros(B, np.float64)
    n = C.c_int32(0)
    _chk(lib().orc_draw_nodes(_p(cand_id), _p(cdf), C.c_int64(len(cand_id)), C.c_int32(B), C.c_uint64(seed),
                              C.c_uint64(it), C.c_uint32(layer), _p(S_next), _p(mult), _p(p_incl), _p(pd), C.byref(n)))
    n = n.value
    return SimpleNamespace(S_next=S_next[:n], mult=mult[:n], p_incl=p_incl[:n], pd=pd[:n], n_next=n)


def sampled_adjacency(g, rows, draw, adj_cap=None):
    """Eq. 3 adjacency of the given rows against the drawn set `draw` (from draw_nodes)."""
    rows = np.ascontiguousarray(rows, np.int32)
    if adj_cap is None:
        r64 = rows.astype(np.int64)
        adj_cap = int((g.rowptr[r64 + 1] - g.rowptr[r64]).sum())
    adj_rowptr = np.zeros(len(rows) + 1, np.int32)
    adj_col = np.zeros(max(adj_cap, 1), np.int32)
    adj_val = np.zeros(max(adj_cap, 1), np.float32)
    nnz = C.c_int64(0)
    S_next = np.ascontiguousarray(draw.S_next, np.int32)
    pd = np.ascontiguousarray(draw.pd, np.float64)
    _chk(lib().orc_sampled_adjacency(C.c_int64(g.n_nodes), _p(g.rowptr), _p(g.colidx), _p(g.val), _p(rows),
                                     C.c_int32(len(rows)), _p(S_next), C.c_int32(len(S_next)), _p(pd),
                                     _p(adj_rowptr), _p(adj_col), _p(adj_val), C.c_int64(adj_cap), C.byref(nnz)))
    nnz = nnz.value
    return SimpleNamespace(adj_rowptr=adj_rowptr, adj_col=adj_col[:nnz], adj_val=adj_val[:nnz], adj_nnz=nnz)


def draw_positions(cdf, B, seed, it, layer):
    cdf = np.ascontiguousarray(cdf, np.uint64)
    pos = np.zeros(B, np.int64)
    _chk(lib().orc_draw_positions(_p(cdf), C.c_int64(len(cdf)), C.c_int32(B), C.c_uint64(seed),
                                  C.c_uint64(it), C.c_uint32(layer), _p(pos)))
    return pos


def remote_count(S_next, lo, hi, part_bounds=None):
    S_next = np.ascontiguousarray(S_next, np.int32)
    n = len(S_next)
    total = C.c_int64(0)
    P = 0 if part_bounds is None else len(part_bounds) - 1
    pb = None if part_bounds is None else np.ascontiguousarray(part_bounds, np.int32)
    per_part = None if part_bounds is None else np.zeros(P, np.int64)
    src_row = np.zeros(max(n, 1), np.int32)
    remote_ids = np.zeros(max(n, 1), np.int32)
    _chk(lib().orc_remote_count(_p(S_next), C.c_int32(n), C.c_int32(lo), C.c_int32(hi), _p(pb),
                                C.c_int32(P), C.byref(total), _p(per_part), _p(src_row), _p(remote_ids)))
    r = total.value
    return SimpleNamespace(remote_total=r, per_part=per_part, src_row=src_row[:n], remote_ids=remote_ids[:r])


def aggregate(adj_rowptr, adj_col, adj_val, X_local, X_remote=None, src_row=None, relu_on_input=False):
    """X_* are 2-D float32 arrays, or uint16 arrays holding bfloat16 bit patterns."""
    adj_rowptr = np.ascontiguousarray(adj_rowptr, np.int32)
    adj_col = np.ascontiguousarray(adj_col, np.int32)
    adj_val = np.ascontiguousarray(adj_val, np.float32)
    nS = len(adj_rowptr) - 1
    X_local = np.ascontiguousarray(X_local)
    dtype = 1 if X_local.dtype == np.uint16 else 0
    if dtype == 0:
        assert X_local.dtype == np.float32
    F = X_local.shape[1]
    if X_remote is not None:
        X_remote = np.ascontiguousarray(X_remote)
        assert X_remote.dtype == X_local.dtype and (X_remote.shape[0] == 0 or X_remote.shape[1] == F)
    sr = None if src_row is None else np.ascontiguousarray(src_row, np.int32)
    Z = np.zeros((nS, F), np.float32)
    _chk(lib().orc_aggregate(_p(adj_rowptr), _p(adj_col), _p(adj_val), C.c_int32(nS),
                             _p(X_local), C.c_int64(F), _p(X_remote), C.c_int64(F), _p(sr),
                             C.c_int32(F), C.c_int(dtype), C.c_int(1 if relu_on_input else 0),
                             _p(Z), C.c_int64(F)))
    return Z


def layer_gemm(Z, W):
    Z = np.ascontiguousarray(Z, np.float32)
    W = np.ascontiguousarray(W, np.float32)
    M, K = Z.shape
    K2, N = W.shape
    assert K == K2
    H = np.zeros((M, N), np.float32)
    _chk(lib().orc_layer_gemm(_p(Z), C.c_int64(K), C.c_int32(M), C.c_int32(K), _p(W), C.c_int64(N),
                              C.c_int32(N), _p(H), C.c_int64(N)))
    return H


def layer_gemm_grad_w(Z, G):
    """dW = Z^T G."""
    Z = np.ascontiguousarray(Z, np.float32)
    G = np.ascontiguousarray(G, np.float32)
    M, K = Z.shape
    M2, N = G.shape
    assert M == M2
    dW = np.zeros((K, N), np.float32)
    _chk(lib().orc_layer_gemm_grad_w(_p(Z), C.c_int64(K), _p(G), C.c_int64(N), C.c_int32(M), C.c_int32(K), C.c_int32(N),
                                     _p(dW), C.c_int64(N)))
    return dW


def layer_gemm_grad_z(G, W):
    """dZ = G W^T (W stored [K x N])."""
    G = np.ascontiguousarray(G, np.float32)
    W = np.ascontiguousarray(W, np.float32)
    M, N = G.shape
    K, N2 = W.shape
    assert N == N2
    dZ = np.zeros((M, K), np.float32)
    _chk(lib().orc_layer_gemm_grad_z(_p(G), C.c_int64(N), C.c_int32(M), C.c_int32(N), _p(W), C.c_int64(N), C.c_int32(K),
                                     _p(dZ), C.c_int64(K)))
    return dZ


def aggregate_grad(adj_rowptr, adj_col, adj_val, n_cols, dZ, H_prev=None):
    """dH_prev = (P~^T dZ) .* [H_prev > 0]; H_prev None: no mask."""
    adj_rowptr = np.ascontiguousarray(adj_rowptr, np.int32)
    adj_col = np.ascontiguousarray(adj_col, np.int32)
    adj_val = np.ascontiguousarray(adj_val, np.float32)
    dZ = np.ascontiguousarray(dZ, np.float32)
    nS, F = dZ.shape
    assert len(adj_rowptr) == nS + 1
    Hp = None if H_prev is None else np.ascontiguousarray(H_prev, np.float32)
    dH = np.zeros((n_cols, F), np.float32)
    _chk(lib().orc_aggregate_grad(_p(adj_rowptr), _p(adj_col), _p(adj_val), C.c_int32(nS), C.c_int32(n_cols), _p(dZ),
                                  C.c_int64(F), C.c_int32(F), _p(Hp), C.c_int64(F), _p(dH), C.c_int64(F)))
    return dH
