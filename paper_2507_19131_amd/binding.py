"""Python binding of libmixaq.so: the same entry points as include/mixaq.h.

Argument marshalling only -- every step of the block runs in the HIP kernels of
the library.  PyTorch supplies device memory (tensors) and streams.  There is
no fallback: if the library is missing, importing the entry points fails.
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmixaq.so")
_lib = None

TOK = 49
QNAMES = ("a_qkv_in", "a_q", "a_k", "a_v", "a_p", "a_proj_in", "a_fc1_in", "a_fc2_in")
TAP_FIELDS = (("a_qkv_in", torch.int8), ("acc_qkv", torch.int32), ("qkv", torch.int8), ("acc_s", torch.int32),
              ("p", torch.int8), ("acc_o", torch.int32), ("a_proj_in", torch.int8), ("acc_proj", torch.int32),
              ("h", torch.float32), ("a_fc1_in", torch.int8), ("acc_fc1", torch.int32), ("a_fc2_in", torch.int8),
              ("acc_fc2", torch.int32), ("y_win", torch.float32))


class MixaqError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("mixaq error %d: %s" % (code, msg))
        self.code = code


class QParam(C.Structure):
    _fields_ = [("scale", C.c_float), ("zero_point", C.c_int32)]


class BlockDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "H", "W", "C", "window", "shift", "heads", "mlp_ratio", "act_bits_high",
                                         "act_bits_low", "weight_bits", "score_mode")] + [("ln_eps", C.c_float)]


class BranchParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta", "b_qkv", "b_proj", "b_fc1",
                                          "b_fc2")] + [(n, QParam) for n in QNAMES]


class SharedParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w_qkv", "w_proj", "w_fc1", "w_fc2", "s_qkv", "s_proj", "s_fc1", "s_fc2",
                                          "rel_pos_bias", "score_gamma", "score_beta")]


class Taps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n, _ in TAP_FIELDS]


class DownsampleDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "B", "H", "W", "C_in", "patch", "N", "act_bits", "weight_bits")] + \
               [("ln_eps", C.c_float)]


class DownsampleParams(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("w", "s_w", "bias", "ln_gamma", "ln_beta")] + [("a_in", QParam)]


def lib_path():
    return _LIB_PATH


def load():
    """Loads libmixaq.so (built by paper_2507_19131_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError("%s not found: build it with `python -m paper_2507_19131_amd.build`" % _LIB_PATH)
        L = C.CDLL(_LIB_PATH)
        L.mixaq_last_error.restype = C.c_char_p
        L.mixaq_keep_count.argtypes = [C.c_int32, C.c_double, C.POINTER(C.c_int32)]
        L.mixaq_block_create.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
        L.mixaq_block_destroy.argtypes = [C.c_void_p]
        L.mixaq_block_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
        L.mixaq_score_windows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.mixaq_select_windows.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.mixaq_block_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_size_t, C.c_void_p]
        L.mixaq_block_forward_taps.argtypes = L.mixaq_block_forward.argtypes + [C.c_void_p]
        L.mixaq_block_forward_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.mixaq_select_windows3.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                            C.c_void_p]
        L.mixaq_block_forward_pruned.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                                 C.c_void_p, C.c_size_t, C.c_void_p]
        L.mixaq_block_forward_profile.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                                  C.c_void_p, C.c_size_t, C.c_void_p, C.c_int32, C.POINTER(C.c_float)]
        L.mixaq_block_forward_scored.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                                 C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.mixaq_stage_forward.argtypes = [C.POINTER(C.c_void_p), C.c_int32, C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.mixaq_downsample_out_shape.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.mixaq_downsample_create.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
        L.mixaq_downsample_destroy.argtypes = [C.c_void_p]
        L.mixaq_downsample_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.mixaq_downsample_forward_taps.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.mixaq_block_set_fused.argtypes = [C.c_void_p, C.c_int32]
        L.mixaq_kernel_name.restype = C.c_char_p
        L.mixaq_kernel_name.argtypes = [C.c_int32]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise MixaqError(rc, load().mixaq_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def make_desc(spec, shift=None):
    """spec: any object with the descriptor's field names (e.g. synth.BlockSpec)."""
    return BlockDesc(spec.B, spec.H, spec.W, spec.C, spec.window, spec.shift if shift is None else shift, spec.heads,
                     spec.mlp_ratio, spec.act_bits_high, spec.act_bits_low, spec.weight_bits, spec.score_mode,
                     spec.ln_eps)


def mixaq_version():
    return load().mixaq_version()


def mixaq_num_windows(desc):
    n = C.c_int32()
    _check(load().mixaq_num_windows(C.byref(desc), C.byref(n)))
    return n.value


def mixaq_keep_count(nW, keep_ratio):
    k = C.c_int32()
    _check(load().mixaq_keep_count(nW, keep_ratio, C.byref(k)))
    return k.value


def mixaq_block_create(desc, shared, branches, stream=None):
    """shared / branches: objects whose attributes are CUDA tensors (see to_device);
    branches[i].q maps quantizer name -> (scale, zero_point).  Returns an opaque handle."""
    sp = SharedParams(*[_ptr(getattr(shared, n)) for n, _ in SharedParams._fields_])
    arr = (BranchParams * 2)()
    for i, b in enumerate(branches):
        for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta", "b_qkv", "b_proj", "b_fc1", "b_fc2"):
            setattr(arr[i], n, _ptr(getattr(b, n)))
        for n in QNAMES:
            setattr(arr[i], n, QParam(b.q[n][0], b.q[n][1]))
    out = C.c_void_p()
    _check(load().mixaq_block_create(C.byref(desc), C.byref(sp), arr, _stream(stream), C.byref(out)))
    return out


def mixaq_block_destroy(blk):
    _check(load().mixaq_block_destroy(blk))


def mixaq_block_workspace_bytes(blk):
    n = C.c_size_t()
    _check(load().mixaq_block_workspace_bytes(blk, C.byref(n)))
    return n.value


def mixaq_score_windows(blk, x, scores, stream=None):
    _check(load().mixaq_score_windows(blk, _ptr(x), _ptr(scores), _stream(stream)))
    return scores


def mixaq_select_windows(scores, B, nW, k_high, reverse, perm, stream=None):
    _check(load().mixaq_select_windows(_ptr(scores), B, nW, k_high, reverse, _ptr(perm), _stream(stream)))
    return perm


def mixaq_select_windows3(scores, B, nW, k_high, k_low, reverse, perm, stream=None):
    _check(load().mixaq_select_windows3(_ptr(scores), B, nW, k_high, k_low, reverse, _ptr(perm), _stream(stream)))
    return perm


def mixaq_block_forward_pruned(blk, x, perm, k_high, k_low, y, workspace, stream=None):
    _check(load().mixaq_block_forward_pruned(blk, _ptr(x), _ptr(perm), k_high, k_low, _ptr(y), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream)))
    return y


def mixaq_block_forward(blk, x, perm, k_high, y, workspace, stream=None):
    _check(load().mixaq_block_forward(blk, _ptr(x), _ptr(perm), k_high, _ptr(y), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream)))
    return y


def mixaq_block_forward_static(blk, x, perm, k_high, y, stream=None):
    """The block on the library's static scratch: no workspace argument, nothing allocated."""
    _check(load().mixaq_block_forward_static(blk, _ptr(x), _ptr(perm), k_high, _ptr(y), _stream(stream)))
    return y


def mixaq_block_forward_taps(blk, x, perm, k_high, y, workspace, taps, stream=None):
    """taps: dict name -> CUDA tensor (missing names are skipped)."""
    tp = Taps(*[_ptr(taps.get(n)) for n, _ in TAP_FIELDS])
    _check(load().mixaq_block_forward_taps(blk, _ptr(x), _ptr(perm), k_high, _ptr(y), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream(stream), C.byref(tp)))
    return y


NUM_KERNELS = 11


def _darr(values):
    return (C.c_double * len(values))(*[float(v) for v in values])


def mixaq_equivalent_act_bits(gmacs, c_gmacs, compress_ratio, prune_ratio, act_bits_base):
    out = C.c_double()
    L = load()
    L.mixaq_equivalent_act_bits.argtypes = [C.c_int32, C.c_void_p, C.c_double, C.c_void_p, C.c_void_p, C.c_double,
                                            C.POINTER(C.c_double)]
    _check(L.mixaq_equivalent_act_bits(len(gmacs), _darr(gmacs), float(c_gmacs), _darr(compress_ratio),
                                       _darr(prune_ratio) if prune_ratio is not None else None, float(act_bits_base),
                                       C.byref(out)))
    return out.value


def mixaq_bops_tera(total_gmacs, act_bits, other_operand_bits=32.0):
    out = C.c_double()
    L = load()
    L.mixaq_bops_tera.argtypes = [C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double)]
    _check(L.mixaq_bops_tera(float(total_gmacs), float(act_bits), float(other_operand_bits), C.byref(out)))
    return out.value


def mixaq_sample_ratios(n, s_min, s_max, upper, uniforms):
    """Returns (ratios list, number of uniforms consumed)."""
    L = load()
    L.mixaq_sample_ratios.argtypes = [C.c_int32, C.c_double, C.c_double, C.c_double, C.c_void_p, C.c_size_t,
                                      C.POINTER(C.c_size_t), C.c_void_p]
    out = (C.c_double * n)()
    used = C.c_size_t()
    u = np.ascontiguousarray(uniforms, dtype=np.float64)
    _check(L.mixaq_sample_ratios(n, s_min, s_max, upper, C.c_void_p(u.ctypes.data), u.size, C.byref(used), out))
    return list(out), used.value


def mixaq_block_set_fused(blk, enable):
    _check(load().mixaq_block_set_fused(blk, int(enable)))


def mixaq_kernel_name(i):
    return load().mixaq_kernel_name(i).decode()


def mixaq_block_forward_scored(blk, x, scores, k_high, k_low, y, workspace, perm_out=None, stream=None):
    _check(load().mixaq_block_forward_scored(blk, _ptr(x), _ptr(scores), k_high, k_low, _ptr(y), _ptr(perm_out), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream)))
    return y


def mixaq_stage_forward(blocks, x, k_high, k_low, y, tmp, scores, perm, workspace, stream=None):
    """blocks: list of handles; k_high / k_low: one int per block pair (k_low None = no pruning)."""
    n = len(blocks)
    handles = (C.c_void_p * n)(*[b.value if isinstance(b, C.c_void_p) else b for b in blocks])
    kh = (C.c_int32 * len(k_high))(*[int(v) for v in k_high])
    kl = (C.c_int32 * len(k_low))(*[int(v) for v in k_low]) if k_low is not None else None
    _check(load().mixaq_stage_forward(handles, n, _ptr(x), kh, kl, _ptr(y), _ptr(tmp), _ptr(scores), _ptr(perm), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream)))
    return y


def mixaq_block_forward_profile(blk, x, perm, k_high, y, workspace, repeats=1, stream=None, scores=None):
    """One forward with HIP events around every kernel (each launched `repeats` times);
    returns {kernel name: mean milliseconds}."""
    ms = (C.c_float * NUM_KERNELS)()
    _check(load().mixaq_block_forward_profile(blk, _ptr(x), _ptr(perm), _ptr(scores), k_high, _ptr(y), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream(stream), int(repeats), ms))
    return {mixaq_kernel_name(i): float(ms[i]) for i in range(NUM_KERNELS)}


def make_downsample_desc(spec):
    """spec: synth.DownSpec (or any object with the same fields)."""
    return DownsampleDesc(spec.kind, spec.B, spec.H, spec.W, spec.C_in, spec.patch, spec.N, spec.act_bits, spec.weight_bits,
                          spec.ln_eps)


def mixaq_downsample_out_shape(desc):
    ho, wo, k = C.c_int32(), C.c_int32(), C.c_int32()
    _check(load().mixaq_downsample_out_shape(C.byref(desc), C.byref(ho), C.byref(wo), C.byref(k)))
    return ho.value, wo.value, k.value


def mixaq_downsample_create(desc, params):
    """params: object with CUDA tensors w, s_w, bias (or None), ln_gamma, ln_beta and a_in = (scale, zero_point)."""
    pp = DownsampleParams(_ptr(params.w), _ptr(params.s_w), _ptr(params.bias), _ptr(params.ln_gamma), _ptr(params.ln_beta),
                          QParam(params.a_in[0], params.a_in[1]))
    out = C.c_void_p()
    _check(load().mixaq_downsample_create(C.byref(desc), C.byref(pp), C.byref(out)))
    return out


def mixaq_downsample_destroy(h):
    _check(load().mixaq_downsample_destroy(h))


def mixaq_downsample_forward(h, x, y, stream=None):
    _check(load().mixaq_downsample_forward(h, _ptr(x), _ptr(y), _stream(stream)))
    return y


def mixaq_downsample_forward_taps(h, x, y, tap_codes=None, tap_acc=None, stream=None):
    _check(load().mixaq_downsample_forward_taps(h, _ptr(x), _ptr(y), _stream(stream), _ptr(tap_codes), _ptr(tap_acc)))
    return y


def downsample_to_device(inp, device="cuda:0"):
    """Copies the numpy arrays of a synth.DownInputs to the device."""
    bag = _Bag()
    for n in ("w", "s_w", "bias", "ln_gamma", "ln_beta"):
        v = getattr(inp, n)
        setattr(bag, n, None if v is None else torch.from_numpy(np.ascontiguousarray(v)).to(device))
    bag.a_in = inp.a_in
    return bag


# ---------------------------------------------------------------- memory helpers (no arithmetic)
class _Bag:
    pass


def to_device(inputs, device="cuda:0"):
    """Copies the numpy arrays of a synth.BlockInputs to the device; returns (shared, branches)."""
    sh = _Bag()
    for n, _ in SharedParams._fields_:
        a = getattr(inputs.shared, n)
        setattr(sh, n, None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(device))
    brs = []
    for b in inputs.branches:
        d = _Bag()
        for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta", "b_qkv", "b_proj", "b_fc1", "b_fc2"):
            setattr(d, n, torch.from_numpy(np.ascontiguousarray(getattr(b, n))).to(device))
        d.q = dict(b.q)
        brs.append(d)
    return sh, brs


def tap_shapes(spec):
    S, Cc, h, F = spec.B * spec.nW, spec.C, spec.heads, spec.C * spec.mlp_ratio
    return dict(a_qkv_in=(S, TOK, Cc), acc_qkv=(S, TOK, 3 * Cc), qkv=(S, TOK, 3 * Cc), acc_s=(S, h, TOK, TOK),
                p=(S, h, TOK, TOK), acc_o=(S, TOK, Cc), a_proj_in=(S, TOK, Cc), acc_proj=(S, TOK, Cc),
                h=(S, TOK, Cc), a_fc1_in=(S, TOK, Cc), acc_fc1=(S, TOK, F), a_fc2_in=(S, TOK, F),
                acc_fc2=(S, TOK, Cc), y_win=(S, TOK, Cc))


def alloc_taps(spec, names="all", device="cuda:0"):
    shapes = tap_shapes(spec)
    return {n: torch.zeros(shapes[n], dtype=dt, device=device) for n, dt in TAP_FIELDS if names == "all" or n in names}


def alloc_workspace(blk, device="cuda:0"):
    return torch.empty(mixaq_block_workspace_bytes(blk), dtype=torch.uint8, device=device)
