"""ctypes binding of include/eora.h: same names without the eora_ prefix, marshalling only.

Host-side packers take and return numpy arrays.  Device entry points take torch CUDA tensors (used
purely as device memory) and launch on torch's current stream.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libeora.so")


class EoraError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, status_string(status), status))


def lib_path():
    return _LIB_PATH


class QMember(ctypes.Structure):
    """eora_q_member of include/eora.h: one layer of a group that shares x."""
    _fields_ = [(n, ctypes.c_void_p) for n in ("qweight", "scales", "qzeros", "A", "B", "A_scales", "B_scales", "y")] + \
               [("d_out", ctypes.c_int)]


class SpMember(ctypes.Structure):
    """eora_sp_member of include/eora.h: one 2:4 layer of a group that shares x."""
    _fields_ = [(n, ctypes.c_void_p) for n in ("values", "indices", "qtiles", "qmeta", "A", "B", "y")] + [("d_out", ctypes.c_int)]


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libeora.so is not built: run `python paper_2410_21271_amd/build.py` "
                          "(there is no CPU fallback)")
    # torch must own the process's HIP runtime: loading it first makes libeora.so bind to the same
    # libamdhip64 (same soname) instead of bringing in a second runtime whose streams and device
    # pointers would be foreign to torch's.
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    sig = {
        "eora_status_string": (ctypes.c_char_p, [ci]),
        "eora_qweight_bytes": (sz, [ci, ci, ci]),
        "eora_qzeros_bytes": (sz, [ci, ci, ci]),
        "eora_scales_bytes": (sz, [ci, ci, ci]),
        "eora_sp24_values_bytes": (sz, [ci, ci]),
        "eora_sp24_indices_bytes": (sz, [ci, ci]),
        "eora_sp24q4_tiles_bytes": (sz, [ci, ci]),
        "eora_sp24q4_meta_bytes": (sz, [ci, ci]),
        "eora_workspace_bytes": (sz, [ci, ci, ci, ci]),
        "eora_workspace_bytes_group": (sz, [ci, ci, ci, ci]),
        "eora_workspace_init": (ci, [vp, sz, vp]),
        "eora_workspace_error": (ci, [vp, vp]),
        "eora_debug_set_spin_limit": (None, [ci]),
        "eora_debug_set_resident_min_blocks": (None, [ci]),
        "eora_debug_set_factors_route": (None, [ci]),
        "eora_debug_last_launch": (ci, [ctypes.c_char_p, sz]),
        "eora_debug_probe": (ci, [ci, vp, sz, vp, vp]),
        "eora_pack_q": (ci, [vp, vp, vp, ci, ci, ci, ci, vp, vp, vp]),
        "eora_pack_factor_f16": (ci, [vp, ci, ci, vp]),
        "eora_pack_factor_q4": (ci, [vp, vp, ci, ci, vp, vp]),
        "eora_pack_factor_q3": (ci, [vp, vp, ci, ci, vp, vp]),
        "eora_pack_sp24": (ci, [vp, vp, ci, ci, vp, vp]),
        "eora_pack_sp24q4": (ci, [vp, vp, vp, vp, ci, ci, ci, vp, vp]),
        "eora_linear_q": (ci, [vp] * 9 + [ci] * 7 + [vp, sz, vp]),
        "eora_linear_q_static": (ci, [vp] * 9 + [ci] * 7 + [vp]),
        "eora_linear_q_multi": (ci, [vp] * 10 + [ci] * 8 + [vp, sz, vp]),
        "eora_linear_q_group": (ci, [vp, ctypes.POINTER(QMember), ci] + [ci] * 6 + [vp, sz, vp]),
        "eora_linear_sp24_group": (ci, [vp, ctypes.POINTER(SpMember), ci, ci, ci, ci, vp, sz, vp]),
        "eora_linear_sp24": (ci, [vp] * 6 + [ci] * 4 + [vp, sz, vp]),
        "eora_linear_sp24q4": (ci, [vp] * 6 + [ci] * 4 + [vp, sz, vp]),
        "eora_unpack_q": (ci, [vp, vp, vp, vp, ci, ci, ci, ci, vp]),
        "eora_dequant_q": (ci, [vp, vp, vp, vp, ci, ci, ci, ci, vp]),
        "eora_expand_sp24": (ci, [vp, vp, vp, ci, ci, vp]),
        "eora_expand_sp24q4": (ci, [vp, vp, vp, ci, ci, vp]),
        "eora_factors_workspace_bytes": (sz, [ci, ci, ci]),
        "eora_factors_store_f16": (ci, [vp, vp, ci, ci, ci, ci, vp, vp, vp, sz, vp]),
        "eora_factors_store_q": (ci, [vp, vp, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]),
        "eora_factors": (ci, [vp, vp, vp, ci, ci, ci, ci, ctypes.c_double, vp, vp, vp, vp, sz, vp, ctypes.POINTER(ctypes.c_double)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    return L


lib = _load()
EXPORTS = ["eora_status_string", "eora_qweight_bytes", "eora_qzeros_bytes", "eora_scales_bytes",
           "eora_sp24_values_bytes", "eora_sp24_indices_bytes", "eora_workspace_bytes", "eora_workspace_bytes_group", "eora_workspace_init",
           "eora_workspace_error", "eora_debug_set_spin_limit", "eora_pack_q",
           "eora_pack_factor_f16", "eora_pack_factor_q4", "eora_pack_sp24", "eora_linear_q",
           "eora_linear_q_group", "eora_linear_sp24", "eora_unpack_q", "eora_dequant_q", "eora_expand_sp24",
           "eora_sp24q4_tiles_bytes", "eora_sp24q4_meta_bytes", "eora_pack_sp24q4", "eora_linear_sp24q4", "eora_expand_sp24q4",
           "eora_factors_workspace_bytes", "eora_factors", "eora_linear_q_multi", "eora_pack_factor_q3", "eora_factors_store_f16", "eora_factors_store_q", "eora_linear_sp24_group",
           "eora_debug_last_launch", "eora_debug_probe", "eora_linear_q_static", "eora_debug_set_resident_min_blocks", "eora_debug_set_factors_route"]


def status_string(status):
    return lib.eora_status_string(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise EoraError(status, where)


# ------------------------------------------------------------------ sizes
def qweight_bytes(d_in, d_out, w_bits):
    return lib.eora_qweight_bytes(d_in, d_out, w_bits)


def qzeros_bytes(d_in, d_out, group):
    return lib.eora_qzeros_bytes(d_in, d_out, group)


def scales_bytes(d_in, d_out, group):
    return lib.eora_scales_bytes(d_in, d_out, group)


def sp24_values_bytes(d_in, d_out):
    return lib.eora_sp24_values_bytes(d_in, d_out)


def sp24_indices_bytes(d_in, d_out):
    return lib.eora_sp24_indices_bytes(d_in, d_out)


def sp24q4_tiles_bytes(d_in, d_out):
    return lib.eora_sp24q4_tiles_bytes(d_in, d_out)


def sp24q4_meta_bytes(d_in, d_out):
    return lib.eora_sp24q4_meta_bytes(d_in, d_out)


def workspace_bytes(M, d_in, d_out, r):
    return lib.eora_workspace_bytes(M, d_in, d_out, r)


# ------------------------------------------------------------------ host packers (numpy in, numpy out)
def _np_ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def pack_q(codes, zeros, scales, w_bits, group):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float16)
    d_out, d_in = codes.shape
    nq, nz, ns = qweight_bytes(d_in, d_out, w_bits), qzeros_bytes(d_in, d_out, group), scales_bytes(d_in, d_out, group)
    if not (nq and nz and ns) or zeros.shape != (d_out, d_in // group) or scales.shape != zeros.shape:
        raise EoraError(-2, "pack_q")
    qw = np.empty(nq // 4, np.uint32)
    qz = np.empty(nz // 4, np.uint32)
    sc = np.empty(ns // 2, np.float16)
    _check(lib.eora_pack_q(_np_ptr(codes), _np_ptr(zeros), _np_ptr(scales), d_in, d_out, w_bits, group,
                           _np_ptr(qw), _np_ptr(qz), _np_ptr(sc)), "pack_q")
    return qw, qz, sc


def pack_factor_f16(mat):
    mat = np.ascontiguousarray(mat, dtype=np.float16)
    rows, cols = mat.shape
    out = np.empty(rows * cols, np.float16)
    _check(lib.eora_pack_factor_f16(_np_ptr(mat), rows, cols, _np_ptr(out)), "pack_factor_f16")
    return out


def pack_factor_q4(codes, scales):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float16)
    rows, cols = codes.shape
    q = np.empty(rows * cols // 8, np.uint32)
    sc = np.empty(scales.size, np.float16)
    _check(lib.eora_pack_factor_q4(_np_ptr(codes), _np_ptr(scales), rows, cols, _np_ptr(q), _np_ptr(sc)),
           "pack_factor_q4")
    return q, sc


def pack_factor_q3(codes, scales):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float16)
    rows, cols = codes.shape
    q = np.empty(rows * cols * 3 // 32, np.uint32)
    sc = np.empty(scales.size, np.float16)
    _check(lib.eora_pack_factor_q3(_np_ptr(codes), _np_ptr(scales), rows, cols, _np_ptr(q), _np_ptr(sc)),
           "pack_factor_q3")
    return q, sc


def pack_sp24(vals, pos):
    vals = np.ascontiguousarray(vals, dtype=np.float16)
    pos = np.ascontiguousarray(pos, dtype=np.uint8)
    d_out, half = vals.shape
    d_in = 2 * half
    values = np.empty(d_out * half, np.float16)
    indices = np.empty(d_out * d_in // 32, np.uint32)
    _check(lib.eora_pack_sp24(_np_ptr(vals), _np_ptr(pos), d_in, d_out, _np_ptr(values), _np_ptr(indices)),
           "pack_sp24")
    return values, indices


def pack_sp24q4(codes, pos, zeros, scales, group):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    pos = np.ascontiguousarray(pos, dtype=np.uint8)
    zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float16)
    d_out, half = codes.shape
    d_in = 2 * half
    nt, nm = sp24q4_tiles_bytes(d_in, d_out), sp24q4_meta_bytes(d_in, d_out)
    if not (nt and nm) or group <= 0 or d_in % group or pos.shape != codes.shape or zeros.shape != (d_out, d_in // group) \
            or scales.shape != zeros.shape:
        raise EoraError(-2, "pack_sp24q4")
    tiles = np.empty(nt // 4, np.uint32)
    meta = np.empty(nm // 4, np.uint32)
    _check(lib.eora_pack_sp24q4(_np_ptr(codes), _np_ptr(pos), _np_ptr(zeros), _np_ptr(scales), d_in, d_out, group,
                                _np_ptr(tiles), _np_ptr(meta)), "pack_sp24q4")
    return tiles, meta


# ------------------------------------------------------------------ device entry points (torch tensors as memory)
def _dp(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def workspace_init(workspace):
    _check(lib.eora_workspace_init(_dp(workspace), workspace.numel() * workspace.element_size(), _stream()),
           "workspace_init")


def workspace_error(workspace):
    """Synchronises the current stream; returns the status code (0 = no in-kernel wait expired)."""
    return lib.eora_workspace_error(_dp(workspace), _stream())


def debug_set_spin_limit(iterations):
    lib.eora_debug_set_spin_limit(int(iterations))


def debug_set_resident_min_blocks(blocks):
    """Test hook: fewest 16-row blocks of a launch that takes the kernel with x resident in LDS (negative: default)."""
    lib.eora_debug_set_resident_min_blocks(int(blocks))


def debug_set_factors_route(route):
    """Test hook: 1 makes factors() always take the eigendecomposition route, 0 restores the choice by the pivots."""
    lib.eora_debug_set_factors_route(int(route))


def debug_last_launch():
    """Name and template parameters of the layer kernel the most recent forward launch chose (a string)."""
    buf = ctypes.create_string_buffer(160)
    _check(lib.eora_debug_last_launch(buf, len(buf)), "debug_last_launch")
    return buf.value.decode()


def debug_probe(kind, src, nbytes, sink):
    """kind 0: empty launch; kind 1: streaming read of nbytes from src.  Enqueued on the current stream."""
    _check(lib.eora_debug_probe(int(kind), _dp(src), int(nbytes), _dp(sink), _stream()), "debug_probe")


def workspace_bytes_group(M, d_in, r, n_members):
    return lib.eora_workspace_bytes_group(M, d_in, r, n_members)


def new_workspace(M, d_in, d_out, r, n_members=1):
    """Allocate (torch, device memory only) and initialise a workspace for the forward calls."""
    import torch
    nbytes = max(workspace_bytes(M, d_in, d_out, r), workspace_bytes_group(M, d_in, r, n_members))
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    workspace_init(ws)
    return ws


def linear_q(x, qweight, scales, qzeros, A, B, A_scales, B_scales, y, M, d_in, d_out, r, w_bits, group, ab_bits,
             workspace):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.eora_linear_q(_dp(x), _dp(qweight), _dp(scales), _dp(qzeros), _dp(A), _dp(B), _dp(A_scales),
                             _dp(B_scales), _dp(y), M, d_in, d_out, r, w_bits, group, ab_bits,
                             _dp(workspace), ws_bytes, _stream()), "linear_q")


def linear_q_static(x, qweight, scales, qzeros, A, B, A_scales, B_scales, y, M, d_in, d_out, r, w_bits, group, ab_bits):
    _check(lib.eora_linear_q_static(_dp(x), _dp(qweight), _dp(scales), _dp(qzeros), _dp(A), _dp(B), _dp(A_scales),
                                    _dp(B_scales), _dp(y), M, d_in, d_out, r, w_bits, group, ab_bits, _stream()),
           "linear_q_static")


def linear_q_group(x, members, M, d_in, r, w_bits, group, ab_bits, workspace):
    """members: sequence of (qweight, scales, qzeros, A, B, A_scales, B_scales, y, d_out)."""
    arr = (QMember * len(members))()
    for e, m in zip(arr, members):
        (e.qweight, e.scales, e.qzeros, e.A, e.B, e.A_scales, e.B_scales, e.y) = [_dp(t) for t in m[:8]]
        e.d_out = m[8]
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.eora_linear_q_group(_dp(x), arr, len(members), M, d_in, r, w_bits, group, ab_bits,
                                   _dp(workspace), ws_bytes, _stream()), "linear_q_group")


def linear_sp24(x, values, indices, A, B, y, M, d_in, d_out, r, workspace):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.eora_linear_sp24(_dp(x), _dp(values), _dp(indices), _dp(A), _dp(B), _dp(y), M, d_in, d_out, r,
                                _dp(workspace), ws_bytes, _stream()), "linear_sp24")


def linear_sp24q4(x, qtiles, qmeta, A, B, y, M, d_in, d_out, r, workspace):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.eora_linear_sp24q4(_dp(x), _dp(qtiles), _dp(qmeta), _dp(A), _dp(B), _dp(y),
                                  M, d_in, d_out, r, _dp(workspace), ws_bytes, _stream()), "linear_sp24q4")


def unpack_q(qweight, qzeros, codes_u8, zeros_u8, d_in, d_out, w_bits, group):
    _check(lib.eora_unpack_q(_dp(qweight), _dp(qzeros), _dp(codes_u8), _dp(zeros_u8), d_in, d_out, w_bits, group,
                             _stream()), "unpack_q")


def dequant_q(qweight, scales, qzeros, W_f32, d_in, d_out, w_bits, group):
    _check(lib.eora_dequant_q(_dp(qweight), _dp(scales), _dp(qzeros), _dp(W_f32), d_in, d_out, w_bits, group,
                              _stream()), "dequant_q")


def expand_sp24(values, indices, W_f16, d_in, d_out):
    _check(lib.eora_expand_sp24(_dp(values), _dp(indices), _dp(W_f16), d_in, d_out, _stream()), "expand_sp24")


def expand_sp24q4(qtiles, qmeta, W_f32, d_in, d_out):
    _check(lib.eora_expand_sp24q4(_dp(qtiles), _dp(qmeta), _dp(W_f32), d_in, d_out, _stream()), "expand_sp24q4")


def linear_q_multi(x, qweight, scales, qzeros, A_all, B_all, A_scales, B_scales, adapter_of_row, y, M, d_in, d_out, r,
                   n_adapters, w_bits, group, ab_bits, workspace):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.eora_linear_q_multi(_dp(x), _dp(qweight), _dp(scales), _dp(qzeros), _dp(A_all), _dp(B_all), _dp(A_scales),
                                   _dp(B_scales), _dp(adapter_of_row), _dp(y), M, d_in, d_out, r, n_adapters, w_bits, group,
                                   ab_bits, _dp(workspace), ws_bytes, _stream()), "linear_q_multi")


# ------------------------------------------------------------------ calibration (Alg. 1 steps 1-6)
def factors_workspace_bytes(d_in, d_out, r):
    return lib.eora_factors_workspace_bytes(d_in, d_out, r)


def factors(W_f32, W_hat_f32, Xt_f32, B_f64, A_f64, sigma_f64, n_tokens, d_in, d_out, r, eig_floor, workspace, stats=False):
    """stats=True returns the eight counters of eora_factors' `stats` argument as a dict."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = (ctypes.c_double * 8)() if stats else None
    _check(lib.eora_factors(_dp(W_f32), _dp(W_hat_f32), _dp(Xt_f32), n_tokens, d_in, d_out, r, float(eig_floor),
                            _dp(B_f64), _dp(A_f64), _dp(sigma_f64), _dp(workspace), ws_bytes, _stream(), st), "factors")
    if stats:
        return dict(eig_sweeps=int(st[0]), eig_ms=st[1], eig_rotations=st[2], eig_rows=int(st[3]),
                    svd_sweeps=int(st[4]), svd_ms=st[5], svd_rotations=st[6], svd_rows=int(st[7]))


def factors_store_f16(B_f64, A_f64, d_in, d_out, r, balance, A_tiles, B_tiles, scratch):
    nbytes = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _check(lib.eora_factors_store_f16(_dp(B_f64), _dp(A_f64), d_in, d_out, r, int(bool(balance)), _dp(A_tiles), _dp(B_tiles),
                                      _dp(scratch), nbytes, _stream()), "factors_store_f16")


def factors_store_q(B_f64, A_f64, d_in, d_out, r, ab_bits, balance, A_q, A_scales, B_q, B_scales, scratch):
    nbytes = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _check(lib.eora_factors_store_q(_dp(B_f64), _dp(A_f64), d_in, d_out, r, ab_bits, int(bool(balance)), _dp(A_q), _dp(A_scales),
                                    _dp(B_q), _dp(B_scales), _dp(scratch), nbytes, _stream()), "factors_store_q")


def linear_sp24_group(x, members, M, d_in, r, workspace):
    """members: sequence of (values, indices, qtiles, qmeta, A, B, y, d_out); tensors or None."""
    arr = (SpMember * len(members))()
    for i, (values, indices, qtiles, qmeta, A, B, y, d_out) in enumerate(members):
        arr[i] = SpMember(*(None if t is None else t.data_ptr() for t in (values, indices, qtiles, qmeta, A, B, y)), int(d_out))
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.eora_linear_sp24_group(_dp(x), arr, len(members), M, d_in, r, _dp(workspace), ws_bytes, _stream()), "linear_sp24_group")
