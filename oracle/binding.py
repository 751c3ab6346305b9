"""ctypes binding of the fp64 CPU oracle (numpy float64 in, numpy float64 out).

Test infrastructure only.  Argument marshalling; all arithmetic is in sa_oracle.c.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

WIN_SYM_CIRCULAR, WIN_SYM_LINEAR, WIN_ONE_SIDED = 0, 1, 2


class Desc(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("n", C.c_int32),
                ("d", C.c_int32), ("w", C.c_int32), ("window", C.c_int32), ("causal", C.c_int32),
                ("perm_B", C.c_int32), ("perm_H", C.c_int32), ("scale", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def desc(B, Hq, Hkv, n, d, w, window=WIN_SYM_CIRCULAR, causal=1, perm_B=1, perm_H=1, scale=0.0):
    return Desc(B, Hq, Hkv, n, d, w, window, causal, perm_B, perm_H, scale)


def _f64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _perm(c, perm):
    if perm is None:
        return None
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    assert perm.shape == (c.perm_B, c.perm_H, c.n), (perm.shape, (c.perm_B, c.perm_H, c.n))
    return perm


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what} failed with code {rc}")


def sa_fwd(c, Q, K, V, perm=None, want_lse=True):
    qs, ks = (c.B, c.Hq, c.n, c.d), (c.B, c.Hkv, c.n, c.d)
    Q, K, V, perm = _f64(Q, qs), _f64(K, ks), _f64(V, ks), _perm(c, perm)
    Y = np.empty(qs, np.float64)
    L = np.empty(qs[:3], np.float64) if want_lse else None
    _check(lib().orc_sa_fwd(C.byref(c), _p(Q), _p(K), _p(V), _p(perm), _p(Y), _p(L)), "orc_sa_fwd")
    return (Y, L) if want_lse else Y


def sa_fwd_rows(c, Q, K, V, perm, rows):
    qs, ks = (c.B, c.Hq, c.n, c.d), (c.B, c.Hkv, c.n, c.d)
    Q, K, V, perm = _f64(Q, qs), _f64(K, ks), _f64(V, ks), _perm(c, perm)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    Y = np.empty((rows.shape[0], c.d), np.float64)
    L = np.empty((rows.shape[0],), np.float64)
    _check(lib().orc_sa_fwd_rows(C.byref(c), _p(Q), _p(K), _p(V), _p(perm), _p(rows),
                                 C.c_int64(rows.shape[0]), _p(Y), _p(L)), "orc_sa_fwd_rows")
    return Y, L


def visible_count(c, perm=None):
    perm = _perm(c, perm)
    cnt = np.empty((c.B, c.Hq, c.n), np.int64)
    _check(lib().orc_visible_count(C.byref(c), _p(perm), _p(cnt)), "orc_visible_count")
    return cnt


def _gate_shape(c, per_dim):
    return (c.B, c.Hq, c.n, c.d) if per_dim else (c.B, c.Hq, c.n)


def gate_combine(c, per_dim, Ysa, Yswa, gsa, gswa):
    qs = (c.B, c.Hq, c.n, c.d)
    Ysa, Yswa = _f64(Ysa, qs), _f64(Yswa, qs)
    gsa, gswa = _f64(gsa, _gate_shape(c, per_dim)), _f64(gswa, _gate_shape(c, per_dim))
    Y = np.empty(qs, np.float64)
    _check(lib().orc_gate_combine(C.byref(c), int(per_dim), _p(Ysa), _p(Yswa), _p(gsa), _p(gswa),
                                  _p(Y)), "orc_gate_combine")
    return Y


def gated_sa_swa_fwd(sa, swa, per_dim, Q, K, V, perm, gsa, gswa):
    """Returns dict with Y, Ysa, Yswa, LSEsa, LSEswa."""
    qs, ks = (sa.B, sa.Hq, sa.n, sa.d), (sa.B, sa.Hkv, sa.n, sa.d)
    Q, K, V, perm = _f64(Q, qs), _f64(K, ks), _f64(V, ks), _perm(sa, perm)
    gsa, gswa = _f64(gsa, _gate_shape(sa, per_dim)), _f64(gswa, _gate_shape(sa, per_dim))
    out = {k: np.empty(qs, np.float64) for k in ("Y", "Ysa", "Yswa")}
    out.update({k: np.empty(qs[:3], np.float64) for k in ("LSEsa", "LSEswa")})
    _check(lib().orc_gated_sa_swa_fwd(C.byref(sa), C.byref(swa), int(per_dim), _p(Q), _p(K), _p(V),
                                      _p(perm), _p(gsa), _p(gswa), _p(out["Y"]), _p(out["Ysa"]),
                                      _p(out["Yswa"]), _p(out["LSEsa"]), _p(out["LSEswa"])),
           "orc_gated_sa_swa_fwd")
    return out


def sa_bwd(c, Q, K, V, perm, dY):
    qs, ks = (c.B, c.Hq, c.n, c.d), (c.B, c.Hkv, c.n, c.d)
    Q, K, V, dY, perm = _f64(Q, qs), _f64(K, ks), _f64(V, ks), _f64(dY, qs), _perm(c, perm)
    dQ, dK, dV = np.empty(qs, np.float64), np.empty(ks, np.float64), np.empty(ks, np.float64)
    _check(lib().orc_sa_bwd(C.byref(c), _p(Q), _p(K), _p(V), _p(perm), _p(dY), _p(dQ), _p(dK),
                            _p(dV)), "orc_sa_bwd")
    return dQ, dK, dV


def gated_sa_swa_bwd(sa, swa, per_dim, Q, K, V, perm, gsa, gswa, dY):
    """Returns dQ, dK, dV, dgsa, dgswa."""
    qs, ks = (sa.B, sa.Hq, sa.n, sa.d), (sa.B, sa.Hkv, sa.n, sa.d)
    gs = _gate_shape(sa, per_dim)
    Q, K, V, dY, perm = _f64(Q, qs), _f64(K, ks), _f64(V, ks), _f64(dY, qs), _perm(sa, perm)
    gsa, gswa = _f64(gsa, gs), _f64(gswa, gs)
    dQ, dK, dV = np.empty(qs, np.float64), np.empty(ks, np.float64), np.empty(ks, np.float64)
    dga, dgl = np.empty(gs, np.float64), np.empty(gs, np.float64)
    _check(lib().orc_gated_sa_swa_bwd(C.byref(sa), C.byref(swa), int(per_dim), _p(Q), _p(K), _p(V),
                                      _p(perm), _p(gsa), _p(gswa), _p(dY), _p(dQ), _p(dK), _p(dV),
                                      _p(dga), _p(dgl)), "orc_gated_sa_swa_bwd")
    return dQ, dK, dV, dga, dgl


def sa_bwd_dq_rows(c, Q, K, V, perm, dY, rows):
    qs, ks = (c.B, c.Hq, c.n, c.d), (c.B, c.Hkv, c.n, c.d)
    Q, K, V, dY, perm = _f64(Q, qs), _f64(K, ks), _f64(V, ks), _f64(dY, qs), _perm(c, perm)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    dQ = np.empty((rows.shape[0], c.d), np.float64)
    _check(lib().orc_sa_bwd_dq_rows(C.byref(c), _p(Q), _p(K), _p(V), _p(perm), _p(dY), _p(rows),
                                    C.c_int64(rows.shape[0]), _p(dQ)), "orc_sa_bwd_dq_rows")
    return dQ


def sa_bwd_dkv_rows(c, Q, K, V, perm, dY, rows):
    qs, ks = (c.B, c.Hq, c.n, c.d), (c.B, c.Hkv, c.n, c.d)
    Q, K, V, dY, perm = _f64(Q, qs), _f64(K, ks), _f64(V, ks), _f64(dY, qs), _perm(c, perm)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    dK = np.empty((rows.shape[0], c.d), np.float64)
    dV = np.empty((rows.shape[0], c.d), np.float64)
    _check(lib().orc_sa_bwd_dkv_rows(C.byref(c), _p(Q), _p(K), _p(V), _p(perm), _p(dY), _p(rows),
                                     C.c_int64(rows.shape[0]), _p(dK), _p(dV)),
           "orc_sa_bwd_dkv_rows")
    return dK, dV


def gate_bwd(c, per_dim, dY, gsa, gswa, Ysa=None, Yswa=None):
    """Returns (dYsa, dYswa) or, when Ysa/Yswa are given, (dYsa, dYswa, dgsa, dgswa)."""
    qs, gs = (c.B, c.Hq, c.n, c.d), _gate_shape(c, per_dim)
    dY, gsa, gswa = _f64(dY, qs), _f64(gsa, gs), _f64(gswa, gs)
    da, dl = np.empty(qs, np.float64), np.empty(qs, np.float64)
    if Ysa is None:
        _check(lib().orc_gate_bwd(C.byref(c), int(per_dim), _p(dY), _p(gsa), _p(gswa), None, None,
                                  _p(da), _p(dl), None, None), "orc_gate_bwd")
        return da, dl
    Ysa, Yswa = _f64(Ysa, qs), _f64(Yswa, qs)
    dga, dgl = np.empty(gs, np.float64), np.empty(gs, np.float64)
    _check(lib().orc_gate_bwd(C.byref(c), int(per_dim), _p(dY), _p(gsa), _p(gswa), _p(Ysa), _p(Yswa),
                              _p(da), _p(dl), _p(dga), _p(dgl)), "orc_gate_bwd")
    return da, dl, dga, dgl


def gate_proj_fwd(c, Ysa, Yswa, Wsa, Wswa, want_logits=False):
    """Eq. 6 + Eq. 5.  Returns Y, or (Y, logits_sa, logits_swa) with want_logits; Yswa = Wswa = None
    selects the single-path gate."""
    qs, dm = (c.B, c.Hq, c.n, c.d), c.Hq * c.d
    Ysa, Wsa = _f64(Ysa, qs), _f64(Wsa, (dm, dm))
    dual = Yswa is not None
    if dual:
        Yswa, Wswa = _f64(Yswa, qs), _f64(Wswa, (dm, dm))
    Y = np.empty(qs, np.float64)
    La = np.empty(qs, np.float64) if want_logits else None
    Lb = np.empty(qs, np.float64) if want_logits and dual else None
    _check(lib().orc_gate_proj_fwd(C.byref(c), _p(Ysa), _p(Yswa) if dual else None, _p(Wsa),
                                   _p(Wswa) if dual else None, _p(Y), _p(La), _p(Lb)), "orc_gate_proj_fwd")
    return (Y, La, Lb) if want_logits else Y


def gate_proj_bwd(c, Ysa, Yswa, Wsa, Wswa, dY):
    """Returns dict(dYsa, dWsa[, dYswa, dWswa])."""
    qs, dm = (c.B, c.Hq, c.n, c.d), c.Hq * c.d
    Ysa, Wsa, dY = _f64(Ysa, qs), _f64(Wsa, (dm, dm)), _f64(dY, qs)
    dual = Yswa is not None
    if dual:
        Yswa, Wswa = _f64(Yswa, qs), _f64(Wswa, (dm, dm))
    out = {"dYsa": np.empty(qs, np.float64), "dWsa": np.empty((dm, dm), np.float64)}
    if dual:
        out.update(dYswa=np.empty(qs, np.float64), dWswa=np.empty((dm, dm), np.float64))
    _check(lib().orc_gate_proj_bwd(C.byref(c), _p(Ysa), _p(Yswa) if dual else None, _p(Wsa),
                                   _p(Wswa) if dual else None, _p(dY), _p(out["dYsa"]),
                                   _p(out.get("dYswa")), _p(out["dWsa"]), _p(out.get("dWswa"))),
           "orc_gate_proj_bwd")
    return out


def dual_path_fwd(sa, swa, Q, K, V, perm, Wsa, Wswa):
    """Alg. 2 as printed: both attention branches, then Eq. 6 gates and the Eq. 5 sum.
    Returns dict(Y, Ysa, Yswa, LSEsa, LSEswa, Lsa, Lswa) (L* = gate logits)."""
    Ysa, LSEsa = sa_fwd(sa, Q, K, V, perm)
    Yswa, LSEswa = sa_fwd(swa, Q, K, V, None)
    Y, La, Lb = gate_proj_fwd(sa, Ysa, Yswa, Wsa, Wswa, want_logits=True)
    return dict(Y=Y, Ysa=Ysa, Yswa=Yswa, LSEsa=LSEsa, LSEswa=LSEswa, Lsa=La, Lswa=Lb)


def dual_path_bwd(sa, swa, Q, K, V, perm, Wsa, Wswa, dY):
    """Chain rule through dual_path_fwd: the gate stage hands each branch its own output gradient,
    each branch is differentiated on its own (Eq. 4 for the permuted one) and dQ, dK, dV are summed.
    Returns dict(dQ, dK, dV, dWsa, dWswa)."""
    Ysa, _ = sa_fwd(sa, Q, K, V, perm)
    Yswa, _ = sa_fwd(swa, Q, K, V, None)
    g = gate_proj_bwd(sa, Ysa, Yswa, Wsa, Wswa, dY)
    a = sa_bwd(sa, Q, K, V, perm, g["dYsa"])
    b = sa_bwd(swa, Q, K, V, None, g["dYswa"])
    return dict(dQ=a[0] + b[0], dK=a[1] + b[1], dV=a[2] + b[2], dWsa=g["dWsa"], dWswa=g["dWswa"])


def decode_fwd(c, q, K, V, length):
    """Decoding step of Sec. 4.2: one query per (b, hq) over rows 0..length-1 of the caches.
    Returns (Y [B,Hq,d], LSE [B,Hq])."""
    ks = (c.B, c.Hkv, c.n, c.d)
    q, K, V = _f64(q, (c.B, c.Hq, c.d)), _f64(K, ks), _f64(V, ks)
    Y = np.empty((c.B, c.Hq, c.d), np.float64)
    L = np.empty((c.B, c.Hq), np.float64)
    _check(lib().orc_decode_fwd(C.byref(c), _p(q), _p(K), _p(V), C.c_int32(int(length)), _p(Y), _p(L)),
           "orc_decode_fwd")
    return Y, L
