"""CPU-side checks of the GPU library: it loads, exports every declared symbol, and its host
logic (key generation, encryption, decryption, circuit lowering, argument checking) agrees
with the independent oracle.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_1806_03461_amd as T
import workloads
from oracle import circuits as cc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "tfhe_mi355x.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:tfhe|bnn)_[a-z0-9_]+)\s*\(", header))
    assert {"tfhe_keygen", "tfhe_encrypt", "tfhe_decrypt", "tfhe_gate_batch", "tfhe_gate_stream",
            "bnn_dense_encrypted", "bnn_conv_encrypted"} <= declared
    L = T.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(T.EXPORTS)


@pytest.fixture(scope="module")
def small():
    P = T.Params(24, 64, 1, 2, 10, 8, 2, -15, -25)
    return P, T.tfhe_keygen(P, 4242)


def test_keygen_matches_oracle_bit_for_bit(orc, small):
    P, (sk, ck) = small
    K = orc.Keys(orc.Params(*[getattr(P, f) for f, _ in P._fields_]), 4242)
    assert np.array_equal(T.tfhe_export_key(sk, T.KEY_LWE_SK), K.lwe_sk)
    assert np.array_equal(T.tfhe_export_key(sk, T.KEY_TRLWE_SK), K.trlwe_sk)
    assert np.array_equal(T.tfhe_export_key(ck, T.KEY_BK_RAW), K.bk)
    assert np.array_equal(T.tfhe_export_key(ck, T.KEY_KSK_RAW), K.ksk)


def test_keygen_matches_oracle_at_benchmark_parameters(real_keys):
    sk, ck = T.tfhe_keygen(T.default_params(), workloads.KEY_SEED)
    assert np.array_equal(T.tfhe_export_key(sk, T.KEY_LWE_SK), real_keys.lwe_sk)
    assert np.array_equal(T.tfhe_export_key(sk, T.KEY_TRLWE_SK), real_keys.trlwe_sk)
    assert np.array_equal(T.tfhe_export_key(ck, T.KEY_BK_RAW), real_keys.bk)
    assert np.array_equal(T.tfhe_export_key(ck, T.KEY_KSK_RAW), real_keys.ksk)


def test_import_keys_round_trip(orc, small):
    """Exported raw material imported again gives keys that export the same bytes, encrypt to the
    same ciphertexts and decrypt them; a server-side cloud key can be built without any secret."""
    P = small[0]
    sk, ck = T.tfhe_keygen(P, 77)
    parts = [T.tfhe_export_key(sk, T.KEY_LWE_SK), T.tfhe_export_key(sk, T.KEY_TRLWE_SK),
             T.tfhe_export_key(ck, T.KEY_BK_RAW), T.tfhe_export_key(ck, T.KEY_KSK_RAW)]
    sk2, ck2 = T.tfhe_import_keys(P, *parts)
    for a, b in ((sk, sk2), (ck, ck2)):
        assert T.tfhe_get_params(a).n == T.tfhe_get_params(b).n
    assert np.array_equal(T.tfhe_export_key(sk2, T.KEY_TRLWE_SK), parts[1])
    assert np.array_equal(T.tfhe_export_key(ck2, T.KEY_BK_RAW), parts[2])
    assert np.array_equal(T.tfhe_export_key(ck2, T.KEY_KSK_RAW), parts[3])
    bits = np.array([1, 0, 0, 1, 1], np.uint8)
    ct = T.tfhe_encrypt(sk2, 5, bits)
    assert np.array_equal(ct, T.tfhe_encrypt(sk, 5, bits)) and list(T.tfhe_decrypt(sk2, ct)) == list(bits)
    none_sk, only_ck = T.tfhe_import_keys(P, bk_raw=parts[2], ksk_raw=parts[3])
    assert none_sk is None and np.array_equal(T.tfhe_export_key(only_ck, T.KEY_KSK_RAW), parts[3])
    # the oracle's own key material is accepted as well: same formats on both sides
    K = orc.Keys(orc.Params(*[getattr(P, f) for f, _ in P._fields_]), 77)
    sk3, ck3 = T.tfhe_import_keys(P, K.lwe_sk, K.trlwe_sk, K.bk, K.ksk)
    assert np.array_equal(T.tfhe_export_key(ck3, T.KEY_BK_RAW), parts[2])
    bad = parts[0].copy()
    bad[0] = 2
    with pytest.raises(T.TfheError):
        T.tfhe_import_keys(P, bad, parts[1], parts[2], parts[3])
    with pytest.raises(ValueError):
        T.tfhe_import_keys(P, parts[0][:-1], parts[1], parts[2], parts[3])


def test_encrypt_decrypt_match_oracle(real_keys):
    sk, _ = T.tfhe_keygen(T.default_params(), workloads.KEY_SEED)
    bits = np.random.default_rng(1).integers(0, 2, 300).astype(np.uint8)
    ct = T.tfhe_encrypt(sk, 99, bits)
    assert np.array_equal(ct, real_keys.encrypt(bits, 99))
    assert np.array_equal(T.tfhe_decrypt(sk, ct), bits)
    noisy = ct.copy()
    noisy[:, -1] += np.uint32(1 << 27)
    assert np.array_equal(T.tfhe_decrypt(sk, noisy), real_keys.decrypt(noisy))
    for b in (0, 1):
        assert np.array_equal(T.tfhe_trivial(T.default_params(), b), real_keys.trivial(b))
    assert T.tfhe_encrypt(sk, 1, np.zeros(0, np.uint8)).shape == (0, 501)


_INTERN = {}


def canonical(gates, outs, n_wires, n_inputs):
    """A circuit as one structural id per output: independent of wire numbering and of the
    order of a gate's two operands.  Equal sub-circuits get equal ids (hash-consing in a table
    shared by both sides of a comparison)."""
    ident = {}
    for w in range(n_inputs + 2):
        ident[w] = _INTERN.setdefault(("in", w), len(_INTERN))
    pending = None
    for g in gates:                                     # topological order
        a = (ident[int(g["in0"])], int(g["neg0"]))
        b = (ident[int(g["in1"])], int(g["neg1"]))
        if int(g["op"]) == 6:                           # multiplexer: (selector, then) ...
            pending = (a, b)
            continue
        if int(g["op"]) == 7:                           # ... (same selector, else): ordered triple
            assert pending is not None and pending[0] == a
            key = ("mux", a, pending[1], b)
            pending = None
        else:
            key = (int(g["op"]),) + tuple(sorted((a, b)))
        ident[int(g["out"])] = _INTERN.setdefault(key, len(_INTERN))
    return [("const", int(v)) if w < 0 else (ident[int(w)], int(v)) for w, v in outs]


def oracle_outs(outs):
    res = []
    for lit in outs:
        if lit is cc.CONST0:
            res.append((-1, 0))
        elif lit is cc.CONST1:
            res.append((-1, 1))
        else:
            res.append(lit)
    return res


@pytest.mark.parametrize("d,p,sparse,with_T", [(5, 3, False, True), (33, 4, True, True), (64, 2, False, False),
                                               (144, 3, False, True), (100, 5, True, False)])
def test_dense_lowering_is_the_oracle_circuit(d, p, sparse, with_T):
    rng = np.random.default_rng(d + p)
    W = (2 * rng.integers(0, 2, (p, d)) - 1).astype(np.int8)
    if sparse:
        W[rng.random((p, d)) < 0.5] = 0
    Tt = rng.integers(-1, d + 2, p).astype(np.int32) if with_T else None
    gates, outs, nw = T.bnn_dense_lower(d, W, Tt, p, 10)
    cir, o = cc.dense_layer(d, W, Tt, 10)
    assert nw == cir.n_wires and len(gates) == len(cir.gates)
    mine = canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, d)
    theirs = canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, d)
    assert mine == theirs


@pytest.mark.parametrize("d,p", [(6, 3), (40, 4), (144, 2)])
def test_mux_comparator_lowering_is_the_oracle_circuit(d, p):
    rng = np.random.default_rng(d)
    W = rng.choice(np.array([-1, 0, 1], np.int8), (p, d), p=[0.4, 0.2, 0.4])
    Tt = rng.integers(-1, d + 2, p).astype(np.int32)
    gates, outs, nw = T.bnn_dense_lower_opts(d, W, Tt, p, 0, T.LOWER_MUX_COMPARATOR)
    cir, o = cc.dense_layer(d, W, Tt, comparator="mux")
    assert nw == cir.n_wires and len(gates) == len(cir.gates)
    mine = canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, d)
    assert mine == canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, d)
    assert (gates["op"] == T.MUX).sum() == (gates["op"] == T.MUX_ELSE).sum() > 0
    with pytest.raises(T.TfheError):
        T.bnn_dense_lower_opts(d, W, Tt, p, 0, 64)


@pytest.mark.parametrize("d,p", [(2, 2), (7, 5), (33, 4), (144, 3), (784, 2)])
def test_plus_one_lowering_is_the_oracle_circuit(d, p):
    rng = np.random.default_rng(7 * d)
    W = (2 * rng.integers(0, 2, (p, d)) - 1).astype(np.int8)
    if d > 2:
        W[p - 1, 1] = 0                                   # this row falls back to the plain unit
    Tt = rng.integers(-1, d + 2, p).astype(np.int32)
    gates, outs, nw = T.bnn_dense_lower_opts(d, W, Tt, p, 0, T.LOWER_PLUS_ONE)
    cir, o = cc.dense_layer(d, W, Tt, plus_one=True)
    assert nw == cir.n_wires and len(gates) == len(cir.gates)
    mine = canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, d)
    assert mine == canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, d)
    c4 = workloads.cfg4(C=2, H=4, Wd=3, O=4)
    gates, outs, nw = T.bnn_conv_lower_opts(2, 4, 3, c4["K"], c4["T"] // 8, 1, 1, T.LOWER_PLUS_ONE)
    cir, o = cc.conv_layer(2, 4, 3, c4["K"], c4["T"] // 8, 1, 1, plus_one=True)
    assert nw == cir.n_wires
    assert canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, 24) == \
        canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, 24)


@pytest.mark.parametrize("plus_one", [False, True])
def test_shared_gate_lowering_is_the_oracle_circuit(plus_one):
    rng = np.random.default_rng(17)
    d, p = 48, 12
    W = (2 * rng.integers(0, 2, (p, d)) - 1).astype(np.int8)
    Tt = rng.integers(10, 40, p).astype(np.int32)
    flags = T.LOWER_SHARE_GATES | (T.LOWER_PLUS_ONE if plus_one else 0)
    gates, outs, nw = T.bnn_dense_lower_opts(d, W, Tt, p, 0, flags)
    cir, o = cc.dense_layer(d, W, Tt, plus_one=plus_one, share=True)
    unshared = len(cc.dense_layer(d, W, Tt, plus_one=plus_one)[0].gates)
    assert nw == cir.n_wires and len(gates) == len(cir.gates) < unshared
    assert canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, d) == \
        canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, d)
    # no (opcode, unordered literal pair) occurs twice
    keys = {(int(g["op"]),) + tuple(sorted(((int(g["in0"]), int(g["neg0"])), (int(g["in1"]), int(g["neg1"]))))) for g in gates}
    assert len(keys) == len(gates)
    for _ in range(4):
        x = rng.integers(0, 2, d).astype(np.uint8)
        assert np.array_equal(cc.eval_plain(cir, x, o), cc.dense_plain(x, W, Tt))
    c4 = workloads.cfg4(C=2, H=4, Wd=3, O=6)
    gates, outs, nw = T.bnn_conv_lower_opts(2, 4, 3, c4["K"], c4["T"] // 8, 1, 1, flags)
    cir, o = cc.conv_layer(2, 4, 3, c4["K"], c4["T"] // 8, 1, 1, plus_one=plus_one, share=True)
    assert nw == cir.n_wires and len(gates) == len(cir.gates)
    assert canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, 24) == \
        canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, 24)


@pytest.mark.parametrize("d,p", [(1, 2), (5, 3), (16, 3), (37, 4), (144, 2)])
def test_sorting_network_lowering_is_the_oracle_circuit(d, p):
    rng = np.random.default_rng(3 * d)
    W = rng.choice(np.array([-1, 0, 1], np.int8), (p, d), p=[0.45, 0.1, 0.45])
    Tt = rng.integers(-1, d + 2, p).astype(np.int32)
    gates, outs, nw = T.bnn_dense_lower_opts(d, W, Tt, p, 0, T.LOWER_SORTING_NETWORK)
    cir, o = cc.dense_layer(d, W, Tt, comparator="sort")
    assert nw == cir.n_wires and len(gates) == len(cir.gates)
    assert canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, d) == \
        canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, d)
    assert set(np.unique(gates["op"])) <= {T.AND, T.OR}
    with pytest.raises(T.TfheError):
        T.bnn_dense_lower_opts(d, W, Tt, p, 0, T.LOWER_SORTING_NETWORK | T.LOWER_PLUS_ONE)


def test_conv_lowering_is_the_oracle_circuit():
    c4 = workloads.cfg4(C=2, H=4, Wd=5, O=3)
    gates, outs, nw = T.bnn_conv_lower(2, 4, 5, c4["K"], c4["T"] // 8, 1, 1)
    cir, o = cc.conv_layer(2, 4, 5, c4["K"], c4["T"] // 8, 1, 1)
    assert nw == cir.n_wires and len(outs) == 3 * 4 * 5
    mine = canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, 40)
    assert mine == canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, 40)
    gates, outs, nw = T.bnn_conv_lower(2, 4, 5, c4["K"], c4["T"] // 8, 2, 0)
    cir, o = cc.conv_layer(2, 4, 5, c4["K"], c4["T"] // 8, 2, 0)
    assert canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, 40) == \
        canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, 40)


def test_paper_shaped_networks_lower_to_the_oracle_circuits():
    """Cancer FC 90->1, the two Diabetes layers (one neuron of the wide one), and the 10x10
    convolution of the Faces shape on a 12x12 corner of its image."""
    c = workloads.paper_cancer()
    gates, outs, nw = T.bnn_dense_lower(90, c["layers"][0]["W"], None, 1, c["out_bits"])
    cir, o = cc.dense_layer(90, c["layers"][0]["W"], None, c["out_bits"])
    assert len(gates) == len(cir.gates) == 585 and len(outs) == 7
    assert canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, 90) == \
        canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, 90)
    c = workloads.paper_diabetes()
    for L, d, rows, ob in ((c["layers"][0], 1704, slice(3, 4), 0), (c["layers"][1], 10, slice(0, 3), c["out_bits"])):
        W, Tt = L["W"][rows], None if L["T"] is None else L["T"][rows]
        gates, outs, nw = T.bnn_dense_lower(d, W, Tt, W.shape[0], ob)
        cir, o = cc.dense_layer(d, W, Tt, ob)
        assert len(gates) == len(cir.gates)
        assert canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, d) == \
            canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, d)
    f = workloads.paper_faces(channels=2)
    assert [k["K"].shape for k in f["convs"]] == [(2, 1, 10, 10), (2, 2, 10, 10), (2, 2, 10, 10), (2, 2, 10, 10),
                                                  (1, 2, 10, 10)] and f["dense"]["W"].shape == (1, 25)
    L = f["convs"][1]
    gates, outs, nw = T.bnn_conv_lower(2, 12, 12, L["K"], L["T"], 1, 0)
    cir, o = cc.conv_layer(2, 12, 12, L["K"], L["T"], 1, 0)
    assert len(outs) == 2 * 3 * 3 and len(gates) == len(cir.gates)
    assert canonical(gates, [(int(r["wire"]), int(r["value"])) for r in outs], nw, 288) == \
        canonical(cir.gate_array(), oracle_outs(o), cir.n_wires, 288)


def test_threaded_lowering_gives_the_serial_records(monkeypatch):
    """Units lowered by several host threads and appended in order are the very records, wire
    numbers included, of the one-thread loop (dense and convolution, MUX comparator included)."""
    rng = np.random.default_rng(5)
    W = rng.choice(np.array([-1, 0, 1], np.int8), (37, 90), p=[0.45, 0.1, 0.45])
    Tt = rng.integers(20, 60, 37).astype(np.int32)
    c4 = workloads.cfg4(C=3, H=6, Wd=7, O=4)
    results = []
    for threads in ("1", "5"):
        monkeypatch.setenv("TFHE_LOWER_THREADS", threads)
        g1, o1, n1 = T.bnn_dense_lower_opts(90, W, Tt, 37, 0, T.LOWER_MUX_COMPARATOR)
        g2, o2, n2 = T.bnn_dense_lower(90, W, None, 37, 8)
        g3, o3, n3 = T.bnn_conv_lower(3, 6, 7, c4["K"], c4["T"] // 6, 1, 1)
        results.append((g1, o1, n1, g2, o2, n2, g3, o3, n3))
    for a, b in zip(*results):
        assert np.array_equal(a, b)
    assert (results[0][0]["op"] == T.MUX).any() and len(results[0][6]) > 4 * 6 * 7 * 20


def test_benchmark_layer_lowering_counts():
    c3 = workloads.cfg3()
    gates, outs, nw = T.bnn_dense_lower(784, c3["W"], c3["T"], 512)
    assert len(outs) == 512 and 512 * 5435 <= len(gates) <= 512 * 5443
    assert nw == 784 + 2 + len(gates)


def test_argument_errors_are_reported_not_thrown():
    L = T.lib()
    bad = T.Params(500, 1000, 1, 2, 10, 8, 2, -15, -25)          # N not a power of two
    sk, ck = C.c_void_p(), C.c_void_p()
    assert L.tfhe_keygen(C.byref(bad), 1, C.byref(sk), C.byref(ck)) == -2
    assert b"power of two" in L.tfhe_last_error()
    bad = T.Params(0, 1024, 1, 2, 10, 8, 2, -15, -25)
    assert L.tfhe_keygen(C.byref(bad), 1, C.byref(sk), C.byref(ck)) == -2
    assert L.tfhe_keygen(None, 1, C.byref(sk), C.byref(ck)) == -1
    ok = T.Params(8, 16, 1, 2, 10, 8, 2, -15, -25)
    assert L.tfhe_keygen(C.byref(ok), 1, None, None) == -1
    assert L.tfhe_encrypt(None, 1, None, 0, None) == -1
    with pytest.raises(T.TfheError):
        T.bnn_dense_lower(4, np.array([[2, 0, 1, 1]], np.int8), np.array([1], np.int32), 1)
    with pytest.raises(T.TfheError):
        T.bnn_dense_lower(300, np.ones((1, 300), np.int8), None, 1, out_bits=8)   # popcount needs 9 bits
    # parameters the kernels do not support are refused before any device work
    sk2, ck2 = T.tfhe_keygen(ok, 3)
    with pytest.raises(T.TfheError) as e:
        T.tfhe_gate_batch(ck2, "AND", 0, 0, 0, 0, stream=0)
    assert e.value.code == -2
    ln = C.c_size_t(3)
    buf = (C.c_uint32 * 1)()
    assert L.tfhe_export_key(sk2.handle, T.KEY_LWE_SK, buf, C.byref(ln)) == -3 and ln.value == 32


def _plain_gate(op, a, b):
    return {T.NAND: 1 - (a & b), T.AND: a & b, T.OR: a | b, T.NOR: 1 - (a | b), T.XOR: a ^ b, T.XNOR: 1 - (a ^ b)}[op]


def _eval_circuit_bits(gates, nwires, fixed_bits):
    """Plain evaluation of gate records on bits, one wire per index (the definition)."""
    w = np.zeros(nwires, np.int64)
    w[:len(fixed_bits)] = fixed_bits
    g = 0
    while g < len(gates):
        r = gates[g]
        a, b = w[r["in0"]] ^ r["neg0"], w[r["in1"]] ^ r["neg1"]
        if r["op"] == T.MUX:
            e = gates[g + 1]
            w[r["out"]] = b if a else (w[e["in1"]] ^ e["neg1"])
            g += 2
        else:
            w[r["out"]] = _plain_gate(int(r["op"]), int(a), int(b))
            g += 1
    return w


def _asap_levels(gates, nwires):
    depth = np.zeros(nwires, np.int64)
    lv = np.zeros(len(gates), np.int64)
    for g, r in enumerate(gates):
        if r["op"] == T.MUX_ELSE:
            lv[g] = lv[g - 1]
            continue
        l = 1 + max(depth[r["in0"]], depth[r["in1"]])
        if r["op"] == T.MUX:
            l = max(l, 1 + depth[gates[g + 1]["in1"]])
        lv[g] = l
        depth[r["out"]] = l
    return lv


@pytest.mark.parametrize("flags", [T.LOWER_DEFAULT, T.LOWER_MUX_COMPARATOR, T.LOWER_PLUS_ONE | T.LOWER_SHARE_GATES,
                                   T.LOWER_SORTING_NETWORK])
def test_wire_pool_plan_keeps_the_circuit_and_never_reuses_a_live_slot(flags):
    """tfhe_plan_wire_pool (the schedule of the layer calls): run depth by depth -- all reads of a
    depth before its writes, as the two kernels of a launch do -- the renamed records give the
    outputs of the circuit as lowered; no slot written at a depth is read at that depth; fixed
    wires and outputs keep their slots; the pool is smaller than one slot per wire."""
    rng = np.random.default_rng(int(flags) + 3)
    d, p = 23, 9
    W = rng.choice(np.array([-1, 0, 1], np.int8), (p, d), p=[0.47, 0.06, 0.47])
    W[0] = 0
    W[0, 5] = -1                                    # a unit that is one negated input: no gate
    Tt = rng.integers(4, 15, p).astype(np.int32)
    Tt[0], Tt[1] = 1, 0                             # unit 0: that input's negation; unit 1: constant 1
    gates, outs, nw = T.bnn_dense_lower_opts(d, W, Tt, p, 0, flags)
    planned, pouts, pool, depths = T.tfhe_plan_wire_pool(gates, nw, d + 2, outs)
    lv = _asap_levels(gates, nw)
    assert depths == lv.max() and len(planned) == len(gates)
    assert d + 2 < pool < nw and pool <= d + 2 + (gates["op"] != T.MUX_ELSE).sum()
    counts = np.bincount(lv, minlength=depths + 1)
    bounds = np.concatenate([[0], np.cumsum(counts[1:])])
    # the plan is the stable depth sort of the records: same opcodes and flags in that order
    order = np.argsort(lv, kind="stable")
    for f in ("op", "neg0", "neg1"):
        assert np.array_equal(planned[f], gates[f][order])
    for trial in range(8):
        x = rng.integers(0, 2, d)
        fixed = np.concatenate([x, [0, 1]])
        want_w = _eval_circuit_bits(gates, nw, fixed)
        want = [(want_w[o["wire"]] ^ o["value"]) if o["wire"] >= 0 else o["value"] for o in outs]
        slots = np.full(pool, -7, np.int64)
        slots[:d + 2] = fixed
        for l in range(1, depths + 1):
            recs = planned[bounds[l - 1]:bounds[l]]
            reads = set(recs["in0"]) | set(recs["in1"])
            writes = set(recs["out"][recs["op"] != T.MUX_ELSE])
            assert not (reads & writes), l                      # a launch reads its inputs before it writes
            assert min(writes) >= d + 2
            a = slots[recs["in0"]] ^ recs["neg0"]
            b = slots[recs["in1"]] ^ recs["neg1"]
            assert (a >= 0).all() and (b >= 0).all() and (a <= 1).all() and (b <= 1).all()
            res = {}
            for k, r in enumerate(recs):
                if r["op"] == T.MUX:
                    res[int(r["out"])] = int(b[k]) if a[k] else int(b[k + 1])
                elif r["op"] != T.MUX_ELSE:
                    res[int(r["out"])] = _plain_gate(int(r["op"]), int(a[k]), int(b[k]))
            for s, v in res.items():
                slots[s] = v
        got = [(slots[o["wire"]] ^ o["value"]) if o["wire"] >= 0 else o["value"] for o in pouts]
        assert got == want
    # pass-through and constant outputs keep their meaning
    if flags == T.LOWER_DEFAULT:
        assert pouts[0]["wire"] == 5 and pouts[0]["value"] == 1 and pouts[1]["wire"] == -1 and pouts[1]["value"] == 1


def test_wire_pool_of_the_benchmark_layer_is_a_fraction_of_its_wires():
    c3 = workloads.cfg3()
    gates, outs, nw = T.bnn_dense_lower(784, c3["W"][:64], c3["T"][:64], 64)
    planned, pouts, pool, depths = T.tfhe_plan_wire_pool(gates, nw, 786, outs)
    assert depths == 36 and pool < 0.45 * nw
    assert len(set(pouts["wire"])) == 64 and pouts["wire"].min() >= 786      # outputs keep distinct slots


def test_wire_pool_planner_rejects_malformed_circuits():
    """The planner validates like the gate-stream executor: cycles, double writes, broken multiplexer
    pairs, wires out of range, writes to fixed wires and outputs that nothing produces are errors."""
    def rec(op, in0, in1, out, neg0=0, neg1=0):
        return (op, neg0, neg1, 0, in0, in1, out)

    def plan(recs, nwires=8, n_fixed=4, outs=((4, 0),)):
        return T.tfhe_plan_wire_pool(np.array(recs, dtype=T.GATE_DTYPE), nwires, n_fixed,
                                     np.array(list(outs), dtype=T.OUT_DTYPE))

    planned, pouts, pool, depths = plan([rec(T.AND, 0, 1, 4), rec(T.OR, 4, 2, 5)], outs=((5, 1), (2, 0), (-1, 1)))
    assert (pool, depths) == (6, 2) and list(pouts["wire"]) == [5, 2, -1] and list(pouts["value"]) == [1, 0, 1]
    for bad, code in (([rec(T.AND, 0, 5, 4), rec(T.OR, 4, 2, 5)], -2),         # reads a wire written later
                      ([rec(T.AND, 4, 1, 4)], -2),                              # reads its own output
                      ([rec(T.AND, 0, 1, 4), rec(T.OR, 0, 2, 4)], -2),          # wire written twice
                      ([rec(T.AND, 0, 1, 9)], -3),                              # wire out of range
                      ([rec(T.AND, 0, 1, 2)], -2),                              # writes a fixed wire
                      ([rec(T.MUX, 0, 1, 4)], -2),                              # multiplexer without its second record
                      ([rec(T.MUX, 0, 1, 4), rec(T.MUX_ELSE, 3, 2, 4)], -2),    # other selector in the second record
                      ([rec(T.MUX_ELSE, 0, 1, 4)], -2),
                      ([rec(9, 0, 1, 4)], -2),                                  # unknown opcode
                      ([rec(T.AND, 0, 6, 4)], -2)):                             # reads a wire nothing writes
        with pytest.raises(T.TfheError) as e:
            plan(bad)
        assert e.value.code == code, (bad, str(e.value))
    with pytest.raises(T.TfheError) as e:
        plan([rec(T.AND, 0, 1, 4)], outs=((6, 0),))                            # output that nothing produces
    assert e.value.code == -2
    planned, pouts, pool, depths = plan([], outs=((1, 1),))                    # no gates at all
    assert (len(planned), pool, depths) == (0, 4, 0)
