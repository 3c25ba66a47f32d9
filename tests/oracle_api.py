"""ctypes access to the CPU oracle (oracle/liboracle.so) for the tests.

Test infrastructure: marshals numpy arrays into the oracle's C structs.  The
product binding has its own, separate marshalling code.
"""
import ctypes as C
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from oracle import build_oracle  # noqa: E402

_lib = None
TOK = 49


class QParam(C.Structure):
    _fields_ = [("scale", C.c_float), ("zero_point", C.c_int32)]


class Desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "H", "W", "C", "window", "shift", "heads", "mlp_ratio",
                                         "act_bits_high", "act_bits_low", "weight_bits", "score_mode")] + \
               [("ln_eps", C.c_float)]


_FP = C.POINTER(C.c_float)
_I8 = C.POINTER(C.c_int8)
_I32 = C.POINTER(C.c_int32)
QN = ("a_qkv_in", "a_q", "a_k", "a_v", "a_p", "a_proj_in", "a_fc1_in", "a_fc2_in")


class Branch(C.Structure):
    _fields_ = [(n, _FP) for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta", "b_qkv", "b_proj", "b_fc1", "b_fc2")] + \
               [(n, QParam) for n in QN]


class Shared(C.Structure):
    _fields_ = [(n, _I8) for n in ("w_qkv", "w_proj", "w_fc1", "w_fc2")] + \
               [(n, _FP) for n in ("s_qkv", "s_proj", "s_fc1", "s_fc2", "rel_pos_bias", "score_gamma", "score_beta")]


TAP_FIELDS = (("a_qkv_in", np.int8), ("acc_qkv", np.int32), ("qkv", np.int8), ("acc_s", np.int32), ("p", np.int8),
              ("acc_o", np.int32), ("a_proj_in", np.int8), ("acc_proj", np.int32), ("h", np.float32),
              ("a_fc1_in", np.int8), ("acc_fc1", np.int32), ("a_fc2_in", np.int8), ("acc_fc2", np.int32),
              ("y_win", np.float32))


class Taps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n, _ in TAP_FIELDS]


class UBParams(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "H", "W", "C", "window", "shift", "heads", "mlp_ratio", "bits")] + \
               [("ln_eps", C.c_float)] + \
               [(n, _FP) for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta", "b_qkv", "b_proj", "b_fc1", "b_fc2")] + \
               [(n, QParam) for n in QN] + \
               [(n, _I8) for n in ("w_qkv", "w_proj", "w_fc1", "w_fc2")] + \
               [(n, _FP) for n in ("s_qkv", "s_proj", "s_fc1", "s_fc2", "rel_pos_bias")]


def lib():
    global _lib
    if _lib is None:
        # ORACLE_LIBRARY_UNDER_TEST: a separately built copy (the planted-mistake test runs the pins against such copies)
        path = os.environ.get("ORACLE_LIBRARY_UNDER_TEST") or build_oracle.build(force=False)
        L = C.CDLL(path)
        L.orc_exp2.restype = C.c_float
        L.orc_exp2.argtypes = [C.c_float]
        L.orc_gelu.restype = C.c_float
        L.orc_gelu.argtypes = [C.c_float]
        L.orc_quantize.restype = C.c_int32
        L.orc_quantize.argtypes = [C.c_float, C.c_float, C.c_int32, C.c_int32]
        L.orc_keep_count.argtypes = [C.c_int32, C.c_double, _I32]
        _lib = L
    return _lib


def _p(a, typ):
    return a.ctypes.data_as(typ) if a is not None else typ()


def make_desc(spec, shift=None):
    return Desc(spec.B, spec.H, spec.W, spec.C, spec.window, spec.shift if shift is None else shift, spec.heads,
                spec.mlp_ratio, spec.act_bits_high, spec.act_bits_low, spec.weight_bits, spec.score_mode, spec.ln_eps)


def make_shared(sh):
    return Shared(*[_p(getattr(sh, n), _I8) for n in ("w_qkv", "w_proj", "w_fc1", "w_fc2")],
                  *[_p(getattr(sh, n), _FP) for n in ("s_qkv", "s_proj", "s_fc1", "s_fc2", "rel_pos_bias",
                                                     "score_gamma", "score_beta")])


def make_branches(brs):
    arr = (Branch * 2)()
    for i, b in enumerate(brs):
        for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta", "b_qkv", "b_proj", "b_fc1", "b_fc2"):
            setattr(arr[i], n, _p(getattr(b, n), _FP))
        for n in QN:
            setattr(arr[i], n, QParam(b.q[n][0], b.q[n][1]))
    return arr


def tap_shapes(spec):
    S, Cc, h, F = spec.B * spec.nW, spec.C, spec.heads, spec.C * spec.mlp_ratio
    return dict(a_qkv_in=(S, TOK, Cc), acc_qkv=(S, TOK, 3 * Cc), qkv=(S, TOK, 3 * Cc), acc_s=(S, h, TOK, TOK),
                p=(S, h, TOK, TOK), acc_o=(S, TOK, Cc), a_proj_in=(S, TOK, Cc), acc_proj=(S, TOK, Cc),
                h=(S, TOK, Cc), a_fc1_in=(S, TOK, Cc), acc_fc1=(S, TOK, F), a_fc2_in=(S, TOK, F),
                acc_fc2=(S, TOK, Cc), y_win=(S, TOK, Cc))


def num_windows(spec):
    n = C.c_int32()
    d = make_desc(spec)
    assert lib().orc_num_windows(C.byref(d), C.byref(n)) == 0
    return n.value


def keep_count(nW, keep):
    k = C.c_int32()
    rc = lib().orc_keep_count(nW, keep, C.byref(k))
    assert rc == 0, rc
    return k.value


def score_windows(inp, x, shift=None):
    spec = inp.spec
    d, sh = make_desc(spec, shift), make_shared(inp.shared)
    out = np.zeros((spec.B, spec.nW), dtype=np.float64)
    rc = lib().orc_score_windows(C.byref(d), C.byref(sh), _p(x, _FP), out.ctypes.data_as(C.POINTER(C.c_double)))
    assert rc == 0, rc
    return out


def select_windows(scores, k_high, reverse=0, k_low=None):
    B, nW = scores.shape
    perm = np.zeros((B, nW), dtype=np.int32)
    sc = np.ascontiguousarray(scores, dtype=np.float64)
    if k_low is None:
        rc = lib().orc_select_windows(sc.ctypes.data_as(C.POINTER(C.c_double)), B, nW, k_high, reverse, _p(perm, _I32))
    else:
        rc = lib().orc_select_windows3(sc.ctypes.data_as(C.POINTER(C.c_double)), B, nW, k_high, k_low, reverse,
                                       _p(perm, _I32))
    assert rc == 0, rc
    return perm


def block_forward(inp, x, perm, k_high, shift=None, want_taps=(), threads=8, k_low=None):
    """Runs the oracle; returns (y, taps dict).  perm None = score+select inside.
    k_low given: windows beyond k_high+k_low in perm are pruned (features forwarded)."""
    spec = inp.spec
    d, sh, br = make_desc(spec, shift), make_shared(inp.shared), make_branches(inp.branches)
    y = np.full((spec.B, spec.H, spec.W, spec.C), np.nan, dtype=np.float32)
    taps, tp = {}, Taps()
    shapes = tap_shapes(spec)
    for n, dt in TAP_FIELDS:
        if want_taps == "all" or n in want_taps:
            taps[n] = np.zeros(shapes[n], dtype=dt)
            setattr(tp, n, taps[n].ctypes.data)
    x = np.ascontiguousarray(x, dtype=np.float32)
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.int32)
    if k_low is None:
        rc = lib().orc_block_forward(C.byref(d), C.byref(sh), br, _p(x, _FP), _p(perm, _I32), int(k_high), _p(y, _FP),
                                     C.byref(tp) if taps else None, int(threads))
    else:
        rc = lib().orc_block_forward_pruned(C.byref(d), C.byref(sh), br, _p(x, _FP), _p(perm, _I32), int(k_high),
                                            int(k_low), _p(y, _FP), C.byref(tp) if taps else None, int(threads))
    assert rc == 0, rc
    return y, taps


def gather_windows(spec, x, perm, shift=None):
    d = make_desc(spec, shift)
    S = spec.B * spec.nW
    win = np.zeros((S, TOK, spec.C), dtype=np.float32)
    valid = np.zeros((S, TOK), dtype=np.uint8)
    rc = lib().orc_gather_windows(C.byref(d), _p(x, _FP), _p(perm, _I32), _p(win, _FP),
                                  valid.ctypes.data_as(C.POINTER(C.c_uint8)))
    assert rc == 0, rc
    return win, valid


def scatter_windows(spec, win, perm, shift=None):
    d = make_desc(spec, shift)
    y = np.full((spec.B, spec.H, spec.W, spec.C), np.nan, dtype=np.float32)
    rc = lib().orc_scatter_windows(C.byref(d), _p(win, _FP), _p(perm, _I32), _p(y, _FP))
    assert rc == 0, rc
    return y


def uniform_block(inp, x, branch, shift=None):
    """The separately written uniform block with the parameters of one branch."""
    spec, sh, b = inp.spec, inp.shared, inp.branches[branch]
    bits = spec.act_bits_high if branch == 0 else spec.act_bits_low
    P = UBParams(spec.B, spec.H, spec.W, spec.C, spec.window, spec.shift if shift is None else shift, spec.heads,
                 spec.mlp_ratio, bits, spec.ln_eps,
                 *[_p(getattr(b, n), _FP) for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta", "b_qkv", "b_proj", "b_fc1", "b_fc2")],
                 *[QParam(b.q[n][0], b.q[n][1]) for n in QN],
                 *[_p(getattr(sh, n), _I8) for n in ("w_qkv", "w_proj", "w_fc1", "w_fc2")],
                 *[_p(getattr(sh, n), _FP) for n in ("s_qkv", "s_proj", "s_fc1", "s_fc2", "rel_pos_bias")])
    y = np.full((spec.B, spec.H, spec.W, spec.C), np.nan, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    rc = lib().ub_forward(C.byref(P), _p(x, _FP), _p(y, _FP))
    assert rc == 0
    return y


# ---------------------------------------------------------------- layers between stages
class DownDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "B", "H", "W", "C_in", "patch", "N", "act_bits", "weight_bits")] + \
               [("ln_eps", C.c_float)]


class DownParams(C.Structure):
    _fields_ = [("w", _I8), ("s_w", _FP), ("bias", _FP), ("ln_gamma", _FP), ("ln_beta", _FP), ("a_in", QParam)]


def downsample_forward(inp, x, want_taps=False, threads=8):
    """inp: synth.DownInputs; x: [B,H,W,C_in] float32.  Returns (out, codes or None, acc or None)."""
    sp = inp.spec
    d = DownDesc(sp.kind, sp.B, sp.H, sp.W, sp.C_in, sp.patch, sp.N, sp.act_bits, sp.weight_bits, sp.ln_eps)
    keep = [np.ascontiguousarray(inp.w, dtype=np.int8), np.ascontiguousarray(inp.s_w, dtype=np.float32),
            None if inp.bias is None else np.ascontiguousarray(inp.bias, dtype=np.float32),
            np.ascontiguousarray(inp.ln_gamma, dtype=np.float32), np.ascontiguousarray(inp.ln_beta, dtype=np.float32)]
    pr = DownParams(_p(keep[0], _I8), _p(keep[1], _FP), _p(keep[2], _FP) if keep[2] is not None else None,
                    _p(keep[3], _FP), _p(keep[4], _FP), QParam(inp.a_in[0], inp.a_in[1]))
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.shape == (sp.B, sp.H, sp.W, sp.C_in)
    tokens = sp.B * sp.Ho * sp.Wo
    out = np.empty((sp.B, sp.Ho, sp.Wo, sp.N), dtype=np.float32)
    codes = np.empty((tokens, sp.K), dtype=np.int8) if want_taps else None
    acc = np.empty((tokens, sp.N), dtype=np.int32) if want_taps else None
    L = lib()
    L.orc_downsample_forward.argtypes = [C.c_void_p, C.c_void_p, _FP, _FP, C.c_void_p, C.c_void_p, C.c_int32]
    rc = L.orc_downsample_forward(C.byref(d), C.byref(pr), _p(x, _FP), _p(out, _FP),
                                  codes.ctypes.data if want_taps else None, acc.ctypes.data if want_taps else None, threads)
    assert rc == 0, rc
    return out, codes, acc
