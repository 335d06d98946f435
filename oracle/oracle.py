"""ctypes front end of the C oracle (oracle/tfhe_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It shares nothing with the GPU library: it loads its own shared object,
built from its own single C file.
"""
import ctypes as C
import os

import numpy as np

from . import build_oracle

OP = {"NAND": 0, "AND": 1, "OR": 2, "NOR": 3, "XOR": 4, "XNOR": 5, "MUX": 6, "MUX_ELSE": 7}

DOMAIN = {"RAW": 0, "LWE_SK": 1, "TRLWE_SK": 2, "BK_A": 3, "BK_E": 4,
          "KSK_A": 5, "KSK_E": 6, "ENC_A": 7, "ENC_E": 8}


class Params(C.Structure):
    _fields_ = [(k, C.c_int32) for k in
                ("n", "N", "k", "bk_l", "bk_Bgbit", "ks_t", "ks_basebit",
                 "lwe_noise_log2", "bk_noise_log2")]

    def as_tuple(self):
        return tuple(getattr(self, f) for f, _ in self._fields_)


def default_params():
    return Params(500, 1024, 1, 2, 10, 8, 2, -15, -25)


GATE_DTYPE = np.dtype([("op", "u1"), ("neg0", "u1"), ("neg1", "u1"), ("pad", "u1"),
                       ("in0", "<i4"), ("in1", "<i4"), ("out", "<i4")])

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.LIB
        if not os.path.exists(path):
            build_oracle.build()
        _lib = C.CDLL(path)
        u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
        u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
        PP = C.POINTER(Params)
        L = _lib
        L.orc_stream_key.restype = C.c_uint64
        L.orc_stream_key.argtypes = [C.c_uint64, C.c_uint32]
        L.orc_rand.restype = C.c_uint64
        L.orc_rand.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64]
        L.orc_noise.restype = C.c_int64
        L.orc_noise.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_int]
        for f in ("orc_negacyclic_definition", "orc_negacyclic_schoolbook", "orc_negacyclic_karatsuba"):
            getattr(L, f).restype = None
            getattr(L, f).argtypes = [u32p, u32p, u32p, C.c_int]
        L.orc_set_product_method.argtypes = [C.c_int]
        L.orc_mul_by_xpow.restype = None
        L.orc_mul_by_xpow.argtypes = [u32p, C.c_int, u32p, C.c_int]
        L.orc_bk_words.restype = C.c_size_t
        L.orc_bk_words.argtypes = [PP]
        L.orc_ksk_words.restype = C.c_size_t
        L.orc_ksk_words.argtypes = [PP]
        L.orc_check_params.argtypes = [PP]
        L.orc_keygen.argtypes = [PP, C.c_uint64, u32p, u32p, C.c_void_p, C.c_void_p]
        L.orc_encrypt.restype = None
        L.orc_encrypt.argtypes = [PP, u32p, C.c_uint64, u8p, C.c_size_t, u32p]
        L.orc_phase.restype = C.c_uint32
        L.orc_phase.argtypes = [u32p, u32p, C.c_int]
        L.orc_decrypt.restype = None
        L.orc_decrypt.argtypes = [PP, u32p, u32p, C.c_size_t, u8p]
        L.orc_trivial.restype = None
        L.orc_trivial.argtypes = [PP, C.c_int, u32p]
        L.orc_gate_precombine.argtypes = [PP, C.c_int, u32p, C.c_int, u32p, C.c_int, u32p]
        L.orc_modswitch.restype = None
        L.orc_modswitch.argtypes = [PP, u32p, u32p]
        L.orc_acc_init.restype = None
        L.orc_acc_init.argtypes = [PP, C.c_uint32, u32p]
        L.orc_decompose.restype = None
        L.orc_decompose.argtypes = [PP, C.c_uint32, np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")]
        L.orc_external_product.restype = None
        L.orc_external_product.argtypes = [PP, u32p, u32p, u32p]
        L.orc_blind_rotate.restype = None
        L.orc_blind_rotate.argtypes = [PP, u32p, u32p, u32p]
        L.orc_sample_extract.restype = None
        L.orc_sample_extract.argtypes = [PP, u32p, u32p]
        L.orc_key_switch.restype = None
        L.orc_key_switch.argtypes = [PP, u32p, u32p, u32p]
        L.orc_gate.argtypes = [PP, u32p, u32p, C.c_int, u32p, C.c_int, u32p, C.c_int, u32p]
        L.orc_gate_batch.argtypes = [PP, u32p, u32p, C.c_void_p, C.c_size_t, u32p, C.c_int]
        L.orc_bootstrap_extract.restype = None
        L.orc_bootstrap_extract.argtypes = [PP, u32p, u32p, u32p]
        L.orc_mux.argtypes = [PP, u32p, u32p, u32p, C.c_int, u32p, C.c_int, u32p, C.c_int, u32p]
    return _lib


def rand(seed, domain, index):
    return lib().orc_rand(seed, DOMAIN[domain] if isinstance(domain, str) else domain, index)


def noise(seed, domain, index, noise_log2):
    return lib().orc_noise(seed, DOMAIN[domain] if isinstance(domain, str) else domain, index, noise_log2)


def negacyclic(a, b, method="karatsuba"):
    a = np.ascontiguousarray(a, dtype=np.uint32)
    b = np.ascontiguousarray(b, dtype=np.uint32)
    c = np.empty_like(a)
    getattr(lib(), "orc_negacyclic_" + method)(a, b, c, len(a))
    return c


def mul_by_xpow(p, a):
    p = np.ascontiguousarray(p, dtype=np.uint32)
    out = np.empty_like(p)
    lib().orc_mul_by_xpow(p, int(a), out, len(p))
    return out


class Keys:
    """Secret keys plus bootstrapping / key-switching keys for one seed."""

    def __init__(self, params, seed, cloud=True):
        self.P = params
        self.seed = seed
        L = lib()
        if L.orc_check_params(C.byref(params)) != 0:
            raise ValueError("bad parameters")
        self.lwe_sk = np.zeros(params.n, np.uint32)
        self.trlwe_sk = np.zeros(params.N, np.uint32)
        self.bk = self.ksk = None
        bkp = kskp = None
        if cloud:
            self.bk = np.zeros(L.orc_bk_words(C.byref(params)), np.uint32)
            self.ksk = np.zeros(L.orc_ksk_words(C.byref(params)), np.uint32)
            bkp, kskp = self.bk.ctypes.data, self.ksk.ctypes.data
        rc = L.orc_keygen(C.byref(params), seed, self.lwe_sk, self.trlwe_sk, bkp, kskp)
        if rc:
            raise RuntimeError("orc_keygen failed")

    # ---- client side -------------------------------------------------
    def encrypt(self, bits, seed):
        bits = np.ascontiguousarray(bits, dtype=np.uint8).ravel()
        ct = np.empty((bits.size, self.P.n + 1), np.uint32)
        lib().orc_encrypt(C.byref(self.P), self.lwe_sk, seed, bits, bits.size, ct)
        return ct

    def decrypt(self, ct):
        ct = np.ascontiguousarray(ct, dtype=np.uint32).reshape(-1, self.P.n + 1)
        bits = np.empty(ct.shape[0], np.uint8)
        lib().orc_decrypt(C.byref(self.P), self.lwe_sk, ct, ct.shape[0], bits)
        return bits

    def phase(self, ct):
        ct = np.ascontiguousarray(ct, dtype=np.uint32).reshape(-1, self.P.n + 1)
        return np.array([lib().orc_phase(np.ascontiguousarray(r), self.lwe_sk, self.P.n) for r in ct],
                        dtype=np.uint32)

    def trivial(self, bit):
        ct = np.empty(self.P.n + 1, np.uint32)
        lib().orc_trivial(C.byref(self.P), int(bit), ct)
        return ct

    # ---- server side: the gate and its steps -------------------------
    def gate(self, op, c0, c1, neg0=0, neg1=0):
        out = np.empty(self.P.n + 1, np.uint32)
        rc = lib().orc_gate(C.byref(self.P), self.bk, self.ksk, OP[op] if isinstance(op, str) else op,
                            np.ascontiguousarray(c0, np.uint32), neg0,
                            np.ascontiguousarray(c1, np.uint32), neg1, out)
        if rc:
            raise ValueError("bad gate op")
        return out

    def mux(self, s, a, b, negs=0, nega=0, negb=0):
        """s ? a : b  (two blind rotations, one key switch)."""
        out = np.empty(self.P.n + 1, np.uint32)
        f = lambda x: np.ascontiguousarray(x, np.uint32)
        lib().orc_mux(C.byref(self.P), self.bk, self.ksk, f(s), negs, f(a), nega, f(b), negb, out)
        return out

    def bootstrap_extract(self, c):
        ext = np.empty(self.P.N + 1, np.uint32)
        lib().orc_bootstrap_extract(C.byref(self.P), self.bk, np.ascontiguousarray(c, np.uint32), ext)
        return ext

    def precombine(self, op, c0, c1, neg0=0, neg1=0):
        out = np.empty(self.P.n + 1, np.uint32)
        rc = lib().orc_gate_precombine(C.byref(self.P), OP[op] if isinstance(op, str) else op,
                                       np.ascontiguousarray(c0, np.uint32), neg0,
                                       np.ascontiguousarray(c1, np.uint32), neg1, out)
        if rc:
            raise ValueError("bad gate op")
        return out

    def modswitch(self, c):
        bar = np.empty(self.P.n + 1, np.uint32)
        lib().orc_modswitch(C.byref(self.P), np.ascontiguousarray(c, np.uint32), bar)
        return bar

    def acc_init(self, bbar):
        acc = np.empty(2 * self.P.N, np.uint32)
        lib().orc_acc_init(C.byref(self.P), int(bbar), acc)
        return acc

    def decompose(self, x):
        d = np.empty(self.P.bk_l, np.int32)
        lib().orc_decompose(C.byref(self.P), int(x) & 0xFFFFFFFF, d)
        return d

    def bk_row(self, i):
        w = 2 * self.P.bk_l * 2 * self.P.N
        return self.bk[i * w:(i + 1) * w]

    def external_product(self, i, D):
        out = np.empty(2 * self.P.N, np.uint32)
        lib().orc_external_product(C.byref(self.P), np.ascontiguousarray(self.bk_row(i)),
                                   np.ascontiguousarray(D, np.uint32), out)
        return out

    def blind_rotate(self, bar, acc):
        acc = np.array(acc, dtype=np.uint32, copy=True)
        lib().orc_blind_rotate(C.byref(self.P), self.bk, np.ascontiguousarray(bar, np.uint32), acc)
        return acc

    def sample_extract(self, acc):
        ext = np.empty(self.P.N + 1, np.uint32)
        lib().orc_sample_extract(C.byref(self.P), np.ascontiguousarray(acc, np.uint32), ext)
        return ext

    def key_switch(self, ext):
        out = np.empty(self.P.n + 1, np.uint32)
        lib().orc_key_switch(C.byref(self.P), self.ksk, np.ascontiguousarray(ext, np.uint32), out)
        return out

    def trlwe_phase(self, acc):
        """B - A*S for a TRLWE sample stored (mask, body)."""
        N = self.P.N
        return (acc[N:] - negacyclic(acc[:N], self.trlwe_sk)).astype(np.uint32)

    def gate_batch(self, gates, wires, threads=1):
        """Evaluate mutually independent gate records in place on `wires`."""
        gates = np.ascontiguousarray(gates, dtype=GATE_DTYPE)
        assert wires.dtype == np.uint32 and wires.flags.c_contiguous
        rc = lib().orc_gate_batch(C.byref(self.P), self.bk, self.ksk, gates.ctypes.data,
                                  gates.size, wires.reshape(-1), threads)
        if rc:
            raise ValueError("bad gate in batch")

    def run_gates(self, gates, wires, threads=1):
        """Evaluate a topologically ordered gate list level by level (gates of one
        level are independent: Sec. 4 'gates at the same level ... in parallel')."""
        gates = np.ascontiguousarray(gates, dtype=GATE_DTYPE)
        for lv in levelize(gates, wires.shape[0]):
            self.gate_batch(gates[lv], wires, threads)


def levelize(gates, nwires):
    """ASAP levels: level(g) = 1 + max(level of the gates producing its inputs)."""
    depth = np.zeros(nwires, np.int64)
    lv = np.zeros(len(gates), np.int64)
    for i, g in enumerate(gates):
        d = 1 + max(depth[g["in0"]], depth[g["in1"]])
        if g["op"] == OP["MUX"]:                       # both halves of a multiplexer share a level
            d = max(d, 1 + depth[gates[i + 1]["in1"]])
        elif g["op"] == OP["MUX_ELSE"]:
            d = lv[i - 1]
        depth[g["out"]] = d
        lv[i] = d
    return [np.nonzero(lv == d)[0] for d in range(1, int(lv.max(initial=0)) + 1)]
