"""Thin Python binding of libsa's C ABI (include/sa.h): argument marshalling only.

Every step of the path runs inside the HIP library; torch is used for device memory and streams.
There is no fallback: if libsa.so is missing the import of this module fails.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsa.so")

SA_OK, SA_ERR_NULL, SA_ERR_SHAPE, SA_ERR_UNSUPPORTED, SA_ERR_WORKSPACE, SA_ERR_BAD_PERM, SA_ERR_HIP = range(7)
SA_ERR_STATIC_LIMIT = 7
SA_STATIC_SCRATCH_BYTES = 8 << 20
SA_BF16, SA_F32 = 0, 1
SA_WIN_SYM_CIRCULAR, SA_WIN_SYM_LINEAR, SA_WIN_ONE_SIDED = 0, 1, 2
SA_OP_FWD, SA_OP_BWD, SA_OP_GATED_FWD, SA_OP_GATED_BWD, SA_OP_CHECK_PERM = range(5)
SA_OP_GATE_PROJ_BWD, SA_OP_GATE_PROJ_BWD_SINGLE, SA_OP_DUAL_PATH_BWD, SA_OP_SAMPLE_PERM = 5, 6, 7, 8
SA_OP_DECODE = 9
SA_OP_BWD_ROPE = 10

EXPORTS = ("sa_status_string", "sa_workspace_bytes", "sa_check_perm", "sa_fwd", "swa_fwd",
           "gated_sa_swa_fwd", "sa_bwd", "sa_permuted_copy", "sa_gate_proj_fwd",
           "sa_gate_proj_bwd", "sa_sample_perm", "sa_dual_path_fwd", "sa_dual_path_bwd",
           "sa_rope_table", "sa_rope", "sa_fwd_rope", "sa_bwd_rope", "sa_decode_fwd", "sa_decode_fwd_varlen",
           "sa_decode_fwd_static")


class sa_desc(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("n", C.c_int32),
                ("d", C.c_int32), ("w", C.c_int32), ("window", C.c_int32),
                ("causal_orig", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float),
                ("perm_B", C.c_int32), ("perm_H", C.c_int32), ("gate_per_dim", C.c_int32),
                ("gate_dtype", C.c_int32)]


class SaError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (sa_status {status})")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_00754_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, sz, ip = C.c_void_p, C.c_size_t, C.c_void_p
    dp = C.POINTER(sa_desc)
    lib.sa_status_string.restype = C.c_char_p
    lib.sa_status_string.argtypes = [C.c_int]
    lib.sa_workspace_bytes.restype = C.c_size_t
    lib.sa_workspace_bytes.argtypes = [dp, C.c_int]
    lib.sa_check_perm.restype = C.c_int
    lib.sa_check_perm.argtypes = [dp, ip, vp, sz, vp]
    lib.sa_fwd.restype = C.c_int
    lib.sa_fwd.argtypes = [dp, vp, vp, vp, ip, vp, vp, vp, sz, vp]
    lib.sa_permuted_copy.restype = C.c_int
    lib.sa_permuted_copy.argtypes = [dp, vp, vp, vp, ip, vp, vp]
    lib.sa_gate_proj_fwd.restype = C.c_int
    lib.sa_gate_proj_fwd.argtypes = [dp] + [vp] * 8
    lib.sa_gate_proj_bwd.restype = C.c_int
    lib.sa_gate_proj_bwd.argtypes = [dp] + [vp] * 12 + [sz, vp]
    lib.sa_sample_perm.restype = C.c_int
    lib.sa_sample_perm.argtypes = [dp, C.c_uint64, C.c_int32, ip, vp, sz, vp]
    lib.sa_dual_path_fwd.restype = C.c_int
    lib.sa_dual_path_fwd.argtypes = [dp, dp, vp, vp, vp, ip] + [vp] * 10
    lib.sa_dual_path_bwd.restype = C.c_int
    lib.sa_dual_path_bwd.argtypes = [dp, dp, vp, vp, vp, ip] + [vp] * 14 + [vp, sz, vp]
    lib.sa_rope_table.restype = C.c_int
    lib.sa_rope_table.argtypes = [C.c_int32, C.c_int32, C.c_double, C.c_int32, vp, vp]
    lib.sa_fwd_rope.restype = C.c_int
    lib.sa_fwd_rope.argtypes = [dp, vp, vp, vp, ip, vp, C.c_int32, vp, vp, vp]
    lib.sa_bwd_rope.restype = C.c_int
    lib.sa_bwd_rope.argtypes = [dp, vp, vp, vp, ip, vp, C.c_int32, C.c_int32, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.sa_rope.restype = C.c_int
    lib.sa_rope.argtypes = [dp, vp, vp, vp, C.c_int32, C.c_int32, vp, vp, vp]
    lib.sa_decode_fwd.restype = C.c_int
    lib.sa_decode_fwd.argtypes = [dp, vp, vp, vp, C.c_int32, vp, vp, vp, sz, vp]
    lib.sa_decode_fwd_static.restype = C.c_int
    lib.sa_decode_fwd_static.argtypes = [dp, vp, vp, vp, C.c_int32, vp, vp, vp]
    lib.sa_decode_fwd_varlen.restype = C.c_int
    lib.sa_decode_fwd_varlen.argtypes = [dp, vp, vp, vp, ip, C.c_int32, vp, vp, vp, sz, vp]
    lib.swa_fwd.restype = C.c_int
    lib.swa_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.gated_sa_swa_fwd.restype = C.c_int
    lib.gated_sa_swa_fwd.argtypes = [dp, dp, vp, vp, vp, ip, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sa_bwd.restype = C.c_int
    lib.sa_bwd.argtypes = [dp, dp] + [vp] * 17 + [sz, vp]
    return lib


_lib = _load()


def status_string(status: int) -> str:
    return _lib.sa_status_string(int(status)).decode()


def make_desc(B, Hq, Hkv, n, d, w, window=SA_WIN_SYM_CIRCULAR, causal_orig=1, dtype=SA_BF16,
              scale=0.0, perm_B=1, perm_H=1, gate_per_dim=0, gate_dtype=SA_F32) -> sa_desc:
    return sa_desc(B, Hq, Hkv, n, d, w, window, causal_orig, dtype, scale, perm_B, perm_H,
                   gate_per_dim, gate_dtype)


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous(), "libsa takes contiguous tensors"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream) if torch.cuda.is_available() else None


def _check(status, what):
    if status != SA_OK:
        raise SaError(status, what)


def sa_workspace_bytes(desc: sa_desc, op: int) -> int:
    return int(_lib.sa_workspace_bytes(C.byref(desc), int(op)))


def sa_check_perm(desc, perm, ws):
    _check(_lib.sa_check_perm(C.byref(desc), _ptr(perm), _ptr(ws), ws.numel() * ws.element_size(),
                              _stream()), "sa_check_perm")


def sa_fwd(desc, Q, K, V, perm, Y, LSE=None):
    _check(_lib.sa_fwd(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(perm), _ptr(Y), _ptr(LSE),
                       None, 0, _stream()), "sa_fwd")


def sa_sample_perm(desc, seed, layer, perm, ws=None):
    _check(_lib.sa_sample_perm(C.byref(desc), C.c_uint64(int(seed) & (2 ** 64 - 1)), int(layer), _ptr(perm),
                               _ptr(ws), (ws.numel() * ws.element_size()) if ws is not None else 0, _stream()),
           "sa_sample_perm")


def sa_permuted_copy(desc, Q, K, V, perm, Y):
    _check(_lib.sa_permuted_copy(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(perm), _ptr(Y), _stream()),
           "sa_permuted_copy")


def sa_gate_proj_fwd(desc, Y_sa, Y_swa, W_sa, W_swa, Y, G_sa=None, G_swa=None):
    _check(_lib.sa_gate_proj_fwd(C.byref(desc), _ptr(Y_sa), _ptr(Y_swa), _ptr(W_sa), _ptr(W_swa), _ptr(Y),
                                 _ptr(G_sa), _ptr(G_swa), _stream()), "sa_gate_proj_fwd")


def sa_gate_proj_bwd(desc, Y_sa, Y_swa, W_sa, W_swa, G_sa, G_swa, dY, dY_sa, dY_swa, dW_sa, dW_swa, ws):
    _check(_lib.sa_gate_proj_bwd(C.byref(desc), _ptr(Y_sa), _ptr(Y_swa), _ptr(W_sa), _ptr(W_swa), _ptr(G_sa),
                                 _ptr(G_swa), _ptr(dY), _ptr(dY_sa), _ptr(dY_swa), _ptr(dW_sa), _ptr(dW_swa),
                                 _ptr(ws), (ws.numel() * ws.element_size()) if ws is not None else 0,
                                 _stream()), "sa_gate_proj_bwd")


def sa_dual_path_fwd(sa, swa, Q, K, V, perm, W_sa, W_swa, Y, Y_sa, Y_swa, G_sa=None, G_swa=None,
                     LSE_sa=None, LSE_swa=None):
    _check(_lib.sa_dual_path_fwd(C.byref(sa), C.byref(swa), _ptr(Q), _ptr(K), _ptr(V), _ptr(perm), _ptr(W_sa),
                                 _ptr(W_swa), _ptr(Y), _ptr(Y_sa), _ptr(Y_swa), _ptr(G_sa), _ptr(G_swa),
                                 _ptr(LSE_sa), _ptr(LSE_swa), _stream()), "sa_dual_path_fwd")


def sa_dual_path_bwd(sa, swa, Q, K, V, perm, W_sa, W_swa, Y_sa, Y_swa, G_sa, G_swa, LSE_sa, LSE_swa, dY,
                     dQ, dK, dV, dW_sa, dW_swa, ws):
    _check(_lib.sa_dual_path_bwd(C.byref(sa), C.byref(swa), _ptr(Q), _ptr(K), _ptr(V), _ptr(perm), _ptr(W_sa),
                                 _ptr(W_swa), _ptr(Y_sa), _ptr(Y_swa), _ptr(G_sa), _ptr(G_swa), _ptr(LSE_sa),
                                 _ptr(LSE_swa), _ptr(dY), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dW_sa),
                                 _ptr(dW_swa), _ptr(ws), (ws.numel() * ws.element_size()) if ws is not None else 0,
                                 _stream()), "sa_dual_path_bwd")


def sa_fwd_rope(desc, Q, K, V, perm, table, Y, LSE=None, interleaved=0):
    _check(_lib.sa_fwd_rope(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(perm), _ptr(table), interleaved,
                            _ptr(Y), _ptr(LSE), _stream()), "sa_fwd_rope")


def sa_bwd_rope(desc, Q, K, V, perm, table, Y, LSE, dY, dQ, dK, dV, ws, interleaved=0, dk_unrotated=0):
    _check(_lib.sa_bwd_rope(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(perm), _ptr(table), interleaved,
                            dk_unrotated, _ptr(Y), _ptr(LSE), _ptr(dY), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(ws),
                            0 if ws is None else ws.numel() * ws.element_size(), _stream()), "sa_bwd_rope")


def sa_rope_table(n, d, base, pos0, table):
    _check(_lib.sa_rope_table(n, d, float(base), pos0, _ptr(table), _stream()), "sa_rope_table")


def sa_rope(desc, Q, K, table, Q_out, K_out, interleaved=0, inverse=0):
    _check(_lib.sa_rope(C.byref(desc), _ptr(Q), _ptr(K), _ptr(table), interleaved, inverse, _ptr(Q_out),
                        _ptr(K_out), _stream()), "sa_rope")


def sa_decode_fwd(desc, q, K, V, length, Y, LSE, ws):
    _check(_lib.sa_decode_fwd(C.byref(desc), _ptr(q), _ptr(K), _ptr(V), int(length), _ptr(Y), _ptr(LSE), _ptr(ws),
                              (ws.numel() * ws.element_size()) if ws is not None else 0, _stream()),
           "sa_decode_fwd")


def sa_decode_fwd_static(desc, q, K, V, length, Y, LSE):
    _check(_lib.sa_decode_fwd_static(C.byref(desc), _ptr(q), _ptr(K), _ptr(V), int(length), _ptr(Y), _ptr(LSE),
                                     _stream()), "sa_decode_fwd_static")


def sa_decode_fwd_varlen(desc, q, K, V, lens, max_len, Y, LSE, ws):
    _check(_lib.sa_decode_fwd_varlen(C.byref(desc), _ptr(q), _ptr(K), _ptr(V), _ptr(lens), int(max_len), _ptr(Y),
                                     _ptr(LSE), _ptr(ws), (ws.numel() * ws.element_size()) if ws is not None else 0,
                                     _stream()), "sa_decode_fwd_varlen")


def swa_fwd(desc, Q, K, V, Y, LSE=None):
    _check(_lib.swa_fwd(C.byref(desc), _ptr(Q), _ptr(K), _ptr(V), _ptr(Y), _ptr(LSE), None, 0,
                        _stream()), "swa_fwd")


def gated_sa_swa_fwd(sa, swa, Q, K, V, perm, gate_sa, gate_swa, Y, Y_sa=None, Y_swa=None,
                     LSE_sa=None, LSE_swa=None, ws=None):
    _check(_lib.gated_sa_swa_fwd(C.byref(sa), C.byref(swa), _ptr(Q), _ptr(K), _ptr(V), _ptr(perm),
                                 _ptr(gate_sa), _ptr(gate_swa), _ptr(Y), _ptr(Y_sa), _ptr(Y_swa),
                                 _ptr(LSE_sa), _ptr(LSE_swa), _ptr(ws),
                                 (ws.numel() * ws.element_size()) if ws is not None else 0, _stream()),
           "gated_sa_swa_fwd")


def sa_bwd(sa, swa, Q, K, V, perm, gate_sa, gate_swa, Y_sa, Y_swa, LSE_sa, LSE_swa, dY,
           dQ, dK, dV, dgate_sa, dgate_swa, ws):
    swa_ref = C.byref(swa) if swa is not None else None
    _check(_lib.sa_bwd(C.byref(sa), swa_ref, _ptr(Q), _ptr(K), _ptr(V), _ptr(perm), _ptr(gate_sa),
                       _ptr(gate_swa), _ptr(Y_sa), _ptr(Y_swa), _ptr(LSE_sa), _ptr(LSE_swa),
                       _ptr(dY), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dgate_sa), _ptr(dgate_swa),
                       _ptr(ws), (ws.numel() * ws.element_size()) if ws is not None else 0,
                       _stream()), "sa_bwd")


def raw():
    """The ctypes library handle (for host-side tests of the error paths)."""
    return _lib
