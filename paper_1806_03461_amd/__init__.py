"""Python binding of the MI355X TFHE / encrypted-BNN library (include/tfhe_mi355x.h).

Argument marshalling only: every function forwards to the C symbol of the same name in
libtfhe_mi355x.so.  Device buffers are torch tensors (int32, contiguous, on the GPU) or raw
device pointers; the stream defaults to torch's current stream.  There is no CPU fallback:
if the library is missing, importing a symbol raises.
"""
import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtfhe_mi355x.so")

NAND, AND, OR, NOR, XOR, XNOR, MUX, MUX_ELSE = range(8)
OPS = {"NAND": NAND, "AND": AND, "OR": OR, "NOR": NOR, "XOR": XOR, "XNOR": XNOR}
LOWER_DEFAULT, LOWER_MUX_COMPARATOR, LOWER_PLUS_ONE, LOWER_SHARE_GATES, LOWER_SORTING_NETWORK = 0, 1, 2, 4, 8
KEY_LWE_SK, KEY_TRLWE_SK, KEY_BK_RAW, KEY_KSK_RAW = range(4)

GATE_DTYPE = np.dtype([("op", "u1"), ("neg0", "u1"), ("neg1", "u1"), ("pad", "u1"),
                       ("in0", "<i4"), ("in1", "<i4"), ("out", "<i4")])
OUT_DTYPE = np.dtype([("wire", "<i4"), ("value", "<i4")])


class TfheError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"tfhe error {code}: {msg}")
        self.code = code


class Params(C.Structure):
    _fields_ = [(k, C.c_int32) for k in
                ("n", "N", "k", "bk_l", "bk_Bgbit", "ks_t", "ks_basebit",
                 "lwe_noise_log2", "bk_noise_log2")]


class Profile(C.Structure):
    _fields_ = [("blind_rotate_ms", C.c_double), ("key_switch_ms", C.c_double),
                ("blind_rotate_launches", C.c_uint64), ("key_switch_launches", C.c_uint64),
                ("gates", C.c_uint64)]


class LayerStats(C.Structure):
    _fields_ = [("gates", C.c_uint64), ("circuit_wires", C.c_uint64), ("pool_wires", C.c_uint64),
                ("depths", C.c_uint64)]


EXPORTS = ["tfhe_last_error", "tfhe_default_params", "tfhe_keygen", "tfhe_encrypt", "tfhe_decrypt",
           "tfhe_trivial", "tfhe_export_key", "tfhe_import_keys", "tfhe_get_params", "tfhe_free_secret_key",
           "tfhe_free_cloud_key", "tfhe_free_buffer", "tfhe_cloud_key_upload", "tfhe_gate_batch",
           "tfhe_gate_batch_noalloc",
           "tfhe_mux_batch", "tfhe_gate_stream", "bnn_dense_lower", "bnn_dense_lower_opts", "bnn_conv_lower",
           "bnn_conv_lower_opts", "bnn_dense_encrypted", "bnn_dense_encrypted_opts", "bnn_conv_encrypted_opts",
           "bnn_conv_encrypted", "tfhe_profile_enable", "tfhe_profile_read", "tfhe_last_layer_stats", "tfhe_plan_wire_pool",
           "tfhe_measure_fp64_peak",
           "tfhe_rounding_margin_enable", "tfhe_rounding_margin_read"]

_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_1806_03461_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, sz, u64, i32 = C.c_void_p, C.c_size_t, C.c_uint64, C.c_int
        L.tfhe_last_error.restype = C.c_char_p
        L.tfhe_default_params.argtypes = [C.POINTER(Params)]
        L.tfhe_keygen.argtypes = [C.POINTER(Params), u64, C.POINTER(vp), C.POINTER(vp)]
        L.tfhe_encrypt.argtypes = [vp, u64, vp, sz, vp]
        L.tfhe_decrypt.argtypes = [vp, vp, sz, vp]
        L.tfhe_trivial.argtypes = [C.POINTER(Params), i32, vp]
        L.tfhe_export_key.argtypes = [vp, i32, vp, C.POINTER(sz)]
        L.tfhe_import_keys.argtypes = [C.POINTER(Params), vp, vp, vp, vp, C.POINTER(vp), C.POINTER(vp)]
        L.tfhe_get_params.argtypes = [vp, i32, C.POINTER(Params)]
        L.tfhe_free_secret_key.argtypes = [vp]
        L.tfhe_free_secret_key.restype = None
        L.tfhe_free_cloud_key.argtypes = [vp]
        L.tfhe_free_cloud_key.restype = None
        L.tfhe_free_buffer.argtypes = [vp]
        L.tfhe_free_buffer.restype = None
        L.tfhe_cloud_key_upload.argtypes = [vp]
        L.tfhe_gate_batch.argtypes = [vp, i32, vp, vp, vp, sz, vp]
        L.tfhe_gate_batch_noalloc.argtypes = [vp, i32, vp, vp, vp, sz, vp]
        L.tfhe_mux_batch.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.tfhe_gate_stream.argtypes = [vp, vp, sz, vp, sz, vp]
        lower_tail = [C.POINTER(vp), C.POINTER(sz), C.POINTER(vp), C.POINTER(sz), C.POINTER(sz)]
        L.bnn_dense_lower.argtypes = [i32, vp, vp, i32, i32] + lower_tail
        L.bnn_dense_lower_opts.argtypes = [i32, vp, vp, i32, i32, C.c_uint32] + lower_tail
        L.bnn_dense_encrypted_opts.argtypes = [vp, vp, i32, vp, vp, i32, vp, i32, C.c_uint32, vp]
        L.bnn_conv_lower_opts.argtypes = [i32, i32, i32, vp, i32, i32, i32, i32, i32, vp, C.c_uint32] + lower_tail
        L.bnn_conv_encrypted_opts.argtypes = [vp, vp, i32, i32, i32, vp, i32, i32, i32, i32, i32, vp, vp,
                                              C.c_uint32, vp]
        L.bnn_conv_lower.argtypes = [i32, i32, i32, vp, i32, i32, i32, i32, i32, vp] + lower_tail
        L.bnn_dense_encrypted.argtypes = [vp, vp, i32, vp, vp, i32, vp, i32, vp]
        L.bnn_conv_encrypted.argtypes = [vp, vp, i32, i32, i32, vp, i32, i32, i32, i32, i32, vp, vp, vp]
        L.tfhe_last_layer_stats.argtypes = [vp, C.POINTER(LayerStats)]
        L.tfhe_plan_wire_pool.argtypes = [vp, sz, sz, sz, vp, sz, C.POINTER(vp), C.POINTER(sz), C.POINTER(sz)]
        L.tfhe_measure_fp64_peak.argtypes = [vp, vp, C.POINTER(C.c_double)]
        L.tfhe_profile_enable.argtypes = [vp, i32]
        L.tfhe_profile_read.argtypes = [vp, C.POINTER(Profile), i32]
        L.tfhe_rounding_margin_enable.argtypes = [vp, i32]
        L.tfhe_rounding_margin_read.argtypes = [vp, C.POINTER(C.c_double)]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise TfheError(rc, lib().tfhe_last_error().decode())


def default_params():
    p = Params()
    lib().tfhe_default_params(C.byref(p))
    return p


def _dev_ptr(t):
    """Device pointer of a torch tensor (checked) or a raw integer pointer."""
    if isinstance(t, int):
        return t
    if not (t.is_cuda and t.is_contiguous() and t.element_size() == 4):
        raise ValueError("device ciphertext buffers must be contiguous 32-bit CUDA tensors")
    return t.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def _host(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


class SecretKey:
    def __init__(self, handle):
        self.handle = handle

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.tfhe_free_secret_key(self.handle)
            self.handle = None


class CloudKey:
    def __init__(self, handle):
        self.handle = handle

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.tfhe_free_cloud_key(self.handle)
            self.handle = None


def tfhe_keygen(params, seed):
    sk, ck = C.c_void_p(), C.c_void_p()
    _check(lib().tfhe_keygen(C.byref(params), seed, C.byref(sk), C.byref(ck)))
    return SecretKey(sk.value), CloudKey(ck.value)


def tfhe_get_params(key):
    p = Params()
    _check(lib().tfhe_get_params(key.handle, int(isinstance(key, CloudKey)), C.byref(p)))
    return p


def tfhe_encrypt(sk, seed, bits):
    """bits: host array of 0/1 -> numpy uint32 [nbits][n+1]."""
    bits = _host(bits, np.uint8).ravel()
    n = tfhe_get_params(sk).n
    ct = np.empty((bits.size, n + 1), np.uint32)
    _check(lib().tfhe_encrypt(sk.handle, seed, bits.ctypes.data, bits.size, ct.ctypes.data))
    return ct


def tfhe_decrypt(sk, ct):
    n = tfhe_get_params(sk).n
    ct = _host(ct, np.uint32).reshape(-1, n + 1)
    bits = np.empty(ct.shape[0], np.uint8)
    _check(lib().tfhe_decrypt(sk.handle, ct.ctypes.data, ct.shape[0], bits.ctypes.data))
    return bits


def tfhe_trivial(params, bit):
    ct = np.empty(params.n + 1, np.uint32)
    _check(lib().tfhe_trivial(C.byref(params), int(bit), ct.ctypes.data))
    return ct


def tfhe_export_key(key, which):
    ln = C.c_size_t(0)
    _check(lib().tfhe_export_key(key.handle, which, None, C.byref(ln)))
    buf = np.empty(ln.value // 4, np.uint32)
    _check(lib().tfhe_export_key(key.handle, which, buf.ctypes.data, C.byref(ln)))
    return buf


def tfhe_import_keys(params, lwe_sk=None, trlwe_sk=None, bk_raw=None, ksk_raw=None):
    """Key objects from raw material (the arrays tfhe_export_key returns).  Returns (sk, ck);
    sk is None without the two secret arrays, ck is None without the two cloud-key arrays."""
    want_sk = lwe_sk is not None and trlwe_sk is not None
    want_ck = bk_raw is not None and ksk_raw is not None
    arrs = [None if a is None else _host(a, np.uint32).ravel() for a in (lwe_sk, trlwe_sk, bk_raw, ksk_raw)]
    sizes = (params.n, params.N, params.n * 2 * params.bk_l * 2 * params.N,
             params.N * params.ks_t * ((1 << params.ks_basebit) - 1) * (params.n + 1))
    for a, size in zip(arrs, sizes):
        if a is not None and a.size != size:
            raise ValueError(f"key array has {a.size} words, the parameters imply {size}")
    ptrs = [None if a is None else a.ctypes.data for a in arrs]
    sk, ck = C.c_void_p(), C.c_void_p()
    _check(lib().tfhe_import_keys(C.byref(params), ptrs[0], ptrs[1], ptrs[2], ptrs[3],
                                  C.byref(sk) if want_sk else None, C.byref(ck) if want_ck else None))
    return (SecretKey(sk.value) if want_sk else None), (CloudKey(ck.value) if want_ck else None)


def tfhe_cloud_key_upload(ck):
    _check(lib().tfhe_cloud_key_upload(ck.handle))


def tfhe_gate_batch(ck, op, a, b, out, count, stream=None):
    op = OPS[op] if isinstance(op, str) else int(op)
    _check(lib().tfhe_gate_batch(ck.handle, op, _dev_ptr(a), _dev_ptr(b), _dev_ptr(out), count, _stream(stream)))


NOALLOC_MAX_GATES = 4096


def tfhe_gate_batch_noalloc(ck, op, a, b, out, count, stream=None):
    op = OPS[op] if isinstance(op, str) else int(op)
    _check(lib().tfhe_gate_batch_noalloc(ck.handle, op, _dev_ptr(a), _dev_ptr(b), _dev_ptr(out), count,
                                         _stream(stream)))


def tfhe_mux_batch(ck, s, a, b, out, count, stream=None):
    _check(lib().tfhe_mux_batch(ck.handle, _dev_ptr(s), _dev_ptr(a), _dev_ptr(b), _dev_ptr(out), count,
                                _stream(stream)))


def tfhe_gate_stream(ck, gates, wires, nwires, stream=None):
    gates = _host(gates, GATE_DTYPE)
    _check(lib().tfhe_gate_stream(ck.handle, gates.ctypes.data, gates.size, _dev_ptr(wires), nwires,
                                  _stream(stream)))


def _take(ptr, count, dtype):
    n = count.value
    if n == 0:
        arr = np.empty(0, dtype)
    else:
        arr = np.frombuffer((C.c_char * (n * dtype.itemsize)).from_address(ptr.value), dtype=dtype).copy()
    lib().tfhe_free_buffer(ptr)
    return arr


def bnn_dense_lower_opts(d, W, T, p, out_bits=0, flags=0):
    W = _host(W, np.int8)
    Tp = None if T is None else _host(T, np.int32)
    g, o = C.c_void_p(), C.c_void_p()
    ng, no, nw = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().bnn_dense_lower_opts(d, W.ctypes.data, None if Tp is None else Tp.ctypes.data, p, out_bits,
                                      flags, C.byref(g), C.byref(ng), C.byref(o), C.byref(no), C.byref(nw)))
    return _take(g, ng, GATE_DTYPE), _take(o, no, OUT_DTYPE), nw.value


def bnn_dense_lower(d, W, T, p, out_bits=0):
    W = _host(W, np.int8)
    Tp = None if T is None else _host(T, np.int32)
    g, o = C.c_void_p(), C.c_void_p()
    ng, no, nw = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().bnn_dense_lower(d, W.ctypes.data, None if Tp is None else Tp.ctypes.data, p, out_bits,
                                 C.byref(g), C.byref(ng), C.byref(o), C.byref(no), C.byref(nw)))
    return _take(g, ng, GATE_DTYPE), _take(o, no, OUT_DTYPE), nw.value


def bnn_conv_lower(C_, H, Wd, K, T, stride, pad):
    K = _host(K, np.int8)
    T = _host(T, np.int32)
    O, _, kh, kw = K.shape
    g, o = C.c_void_p(), C.c_void_p()
    ng, no, nw = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().bnn_conv_lower(C_, H, Wd, K.ctypes.data, O, kh, kw, stride, pad, T.ctypes.data,
                                C.byref(g), C.byref(ng), C.byref(o), C.byref(no), C.byref(nw)))
    return _take(g, ng, GATE_DTYPE), _take(o, no, OUT_DTYPE), nw.value


def bnn_conv_lower_opts(C_, H, Wd, K, T, stride, pad, flags=0):
    K = _host(K, np.int8)
    T = _host(T, np.int32)
    O, _, kh, kw = K.shape
    g, o = C.c_void_p(), C.c_void_p()
    ng, no, nw = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().bnn_conv_lower_opts(C_, H, Wd, K.ctypes.data, O, kh, kw, stride, pad, T.ctypes.data, flags,
                                     C.byref(g), C.byref(ng), C.byref(o), C.byref(no), C.byref(nw)))
    return _take(g, ng, GATE_DTYPE), _take(o, no, OUT_DTYPE), nw.value


def bnn_conv_encrypted_opts(ck, x, C_, H, Wd, K, T, stride, pad, out, flags=0, stream=None):
    K = _host(K, np.int8)
    T = _host(T, np.int32)
    O, _, kh, kw = K.shape
    _check(lib().bnn_conv_encrypted_opts(ck.handle, _dev_ptr(x), C_, H, Wd, K.ctypes.data, O, kh, kw, stride,
                                         pad, T.ctypes.data, _dev_ptr(out), flags, _stream(stream)))


def bnn_dense_encrypted(ck, x, d, W, T, p, out, out_bits=0, stream=None):
    W = _host(W, np.int8)
    Tp = None if T is None else _host(T, np.int32)
    _check(lib().bnn_dense_encrypted(ck.handle, _dev_ptr(x), d, W.ctypes.data,
                                     None if Tp is None else Tp.ctypes.data, p, _dev_ptr(out), out_bits,
                                     _stream(stream)))


def bnn_dense_encrypted_opts(ck, x, d, W, T, p, out, out_bits=0, flags=0, stream=None):
    W = _host(W, np.int8)
    Tp = None if T is None else _host(T, np.int32)
    _check(lib().bnn_dense_encrypted_opts(ck.handle, _dev_ptr(x), d, W.ctypes.data,
                                          None if Tp is None else Tp.ctypes.data, p, _dev_ptr(out), out_bits,
                                          flags, _stream(stream)))


def bnn_conv_encrypted(ck, x, C_, H, Wd, K, T, stride, pad, out, stream=None):
    K = _host(K, np.int8)
    T = _host(T, np.int32)
    O, _, kh, kw = K.shape
    _check(lib().bnn_conv_encrypted(ck.handle, _dev_ptr(x), C_, H, Wd, K.ctypes.data, O, kh, kw, stride, pad,
                                    T.ctypes.data, _dev_ptr(out), _stream(stream)))


def tfhe_plan_wire_pool(gates, nwires, n_fixed, outs):
    """Depth-sorted records in pool-slot numbers, the rewritten output references, pool size, depths."""
    gates = _host(gates, GATE_DTYPE)
    outs = np.array(outs, dtype=OUT_DTYPE, copy=True)
    planned, pool, depths = C.c_void_p(), C.c_size_t(), C.c_size_t()
    _check(lib().tfhe_plan_wire_pool(gates.ctypes.data, gates.size, nwires, n_fixed, outs.ctypes.data, outs.size,
                                     C.byref(planned), C.byref(pool), C.byref(depths)))
    return _take(planned, C.c_size_t(gates.size), GATE_DTYPE), outs, pool.value, depths.value


def tfhe_last_layer_stats(ck):
    st = LayerStats()
    _check(lib().tfhe_last_layer_stats(ck.handle, C.byref(st)))
    return {f: getattr(st, f) for f, _ in LayerStats._fields_}


def tfhe_profile_enable(ck, on=True):
    _check(lib().tfhe_profile_enable(ck.handle, int(on)))


def tfhe_profile_read(ck, reset=True):
    p = Profile()
    _check(lib().tfhe_profile_read(ck.handle, C.byref(p), int(reset)))
    return {f: getattr(p, f) for f, _ in Profile._fields_}


def tfhe_measure_fp64_peak(ck, stream=None):
    v = C.c_double()
    _check(lib().tfhe_measure_fp64_peak(ck.handle, _stream(stream), C.byref(v)))
    return v.value


def tfhe_rounding_margin_enable(ck, on=True):
    _check(lib().tfhe_rounding_margin_enable(ck.handle, int(on)))


def tfhe_rounding_margin_read(ck):
    v = C.c_double()
    _check(lib().tfhe_rounding_margin_read(ck.handle, C.byref(v)))
    return v.value


# helpers for moving ciphertexts between numpy and torch without reinterpreting values
def to_device(ct):
    import torch
    return torch.from_numpy(np.ascontiguousarray(ct, np.uint32).view(np.int32)).cuda()


def to_host(t):
    return t.detach().cpu().numpy().view(np.uint32)
