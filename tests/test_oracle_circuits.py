"""Pins for the oracle's circuit layer: reduce-tree popcount, comparator chain,
dense / convolution lowering, against integer popcounts, the paper's closed form for
a BNN unit, the gate counts the paper states, and a library correlation."""
import itertools
import os

import numpy as np
import pytest
from scipy.signal import correlate

import workloads
from oracle import circuits as cc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def paper_counts():
    d = {}
    for line in open(os.path.join(GOLD, "paper_gate_counts.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            d[k] = int(v)
    return d


def popcount_bits(m, weights=None):
    cir = cc.Circuit(m)
    w = np.ones(m, np.int8) if weights is None else weights
    outs = cc.neuron(cir, [(i, 0) for i in range(m)], w, None, out_bits=max(1, int(m).bit_length()))
    return cir, outs


# --------------------------------------------------------------------------- popcount tree
@pytest.mark.parametrize("m", range(1, 13))
def test_popcount_tree_exhaustive(m):
    cir, outs = popcount_bits(m)
    for bits in itertools.product((0, 1), repeat=m):
        got = cc.eval_plain(cir, np.array(bits, np.uint8), outs)
        assert sum(int(b) << i for i, b in enumerate(got)) == sum(bits)


@pytest.mark.parametrize("m", [13, 31, 64, 90, 144, 257, 784, 1704])
def test_popcount_tree_random_with_signed_weights(m):
    rng = np.random.default_rng(m)
    w = rng.choice(np.array([-1, 0, 1], np.int8), m, p=[0.4, 0.2, 0.4])
    cir, outs = popcount_bits(m, w)
    for trial in range(6):
        x = (rng.random(m) < (0.5, 0.05, 0.95)[trial % 3]).astype(np.uint8)
        got = cc.eval_plain(cir, x, outs)
        want = int(((x == 1) & (w == 1)).sum() + ((x == 0) & (w == -1)).sum())
        assert sum(int(b) << i for i, b in enumerate(got)) == want
    for x in (np.zeros(m, np.uint8), np.ones(m, np.uint8)):
        got = cc.eval_plain(cir, x, outs)
        want = int(((x == 1) & (w == 1)).sum() + ((x == 0) & (w == -1)).sum())
        assert sum(int(b) << i for i, b in enumerate(got)) == want


def test_adder_gate_counts_match_paper_statement():
    """A half adder is 2 gates; a full-adder cell is 5 gates (the paper's '5k gates per k-bit
    RC adder'); this build's k-bit adder starts with a half adder at bit 0, hence 5k - 3."""
    pc = paper_counts()
    cir = cc.Circuit(2)
    cc.add_numbers(cir, ([(0, 0)], 1), ([(1, 0)], 1))
    assert len(cir.gates) == pc["half_adder_gates"]
    for k in range(2, 9):
        cir = cc.Circuit(2 * k)
        a = ([(i, 0) for i in range(k)], 2**k - 1)
        b = ([(k + i, 0) for i in range(k)], 2**k - 1)
        cc.add_numbers(cir, a, b)
        assert len(cir.gates) == pc["rc_adder_gates_per_bit"] * k - 3


@pytest.mark.parametrize("k", range(1, 11))
def test_tree_gate_count_closed_form_power_of_two(k):
    d = 2**k
    cir, _ = popcount_bits(d)
    want = d + sum((d >> j) * (5 * j - 3) for j in range(2, k + 1))
    assert len(cir.gates) == want


def depth_of(cir):
    depth = np.zeros(cir.n_wires, np.int64)
    for (_, _, _, _, i0, i1, o) in cir.gates:
        depth[o] = 1 + max(depth[i0], depth[i1])
    return int(depth.max())


def test_benchmark_neuron_sizes():
    """Tree sizes / depths of the benchmark's unit circuits; the comparator adds 1..w-1 gates
    and one to w-1 levels (w = bit width of the popcount)."""
    for m, tree, tree_depth, thresholds in ((144, 966, 25, range(55, 90)), (256, 1745, 28, range(96, 161)),
                                            (784, 5434, 35, range(300, 485))):
        cir, _ = popcount_bits(m)
        assert len(cir.gates) == tree and depth_of(cir) == tree_depth
        w = int(m).bit_length()
        for t in thresholds:
            cir = cc.Circuit(m)
            cc.neuron(cir, [(i, 0) for i in range(m)], np.ones(m, np.int8), t)
            assert tree + 1 <= len(cir.gates) <= tree + w - 1
            assert depth_of(cir) == tree_depth + 1          # the chain runs beside the ripple carry


# --------------------------------------------------------------------------- comparator
@pytest.mark.parametrize("m", [1, 2, 3, 5, 8, 13, 31, 32, 33, 64])
def test_threshold_chain_all_S_all_T(m):
    for T in range(-1, m + 3):
        cir = cc.Circuit(m)
        outs = cc.neuron(cir, [(i, 0) for i in range(m)], np.ones(m, np.int8), T)
        for S in range(m + 1):
            x = np.zeros(m, np.uint8)
            x[:S] = 1
            assert cc.eval_plain(cir, x, outs)[0] == (1 if S >= T else 0), (m, T, S)


def test_threshold_chain_gate_budget():
    """At most w-1 two-input gates for a w-bit popcount (Algorithm 1 would use w MUX gates)."""
    for m in (7, 144, 256, 784):
        w = int(m).bit_length()
        base = len(popcount_bits(m)[0].gates)
        for T in range(1, m + 1):
            cir = cc.Circuit(m)
            cc.neuron(cir, [(i, 0) for i in range(m)], np.ones(m, np.int8), T)
            assert len(cir.gates) - base <= w - 1


# --------------------------------------------------------------------------- layers
def test_threshold_form_equals_paper_sign_form():
    """[S >= ceil((d-b)/2)] equals sign(2 S - d + b) with sign(0) = +1 (Sec. 3.2, step 4)."""
    rng = np.random.default_rng(0)
    for _ in range(300):
        d = int(rng.integers(1, 200))
        b = int(rng.integers(-d - 3, d + 4))
        w = 2 * rng.integers(0, 2, d) - 1
        x = rng.integers(0, 2, d).astype(np.uint8)
        z = 1 if int((w * (2 * x.astype(int) - 1)).sum()) + b >= 0 else 0
        T = -((b - d) // 2)                       # ceil((d - b) / 2)
        assert cc.dense_plain(x, w.reshape(1, d).astype(np.int8), np.array([T]))[0] == z


@pytest.mark.parametrize("d,p,sparse", [(9, 5, False), (90, 3, False), (64, 6, True), (200, 4, True)])
def test_dense_circuit_equals_integer_layer(d, p, sparse):
    rng = np.random.default_rng(d * p)
    W = (2 * rng.integers(0, 2, (p, d)) - 1).astype(np.int8)
    if sparse:
        W[rng.random((p, d)) < 0.5] = 0
    m = (W != 0).sum(axis=1)
    T = np.array([rng.integers(-1, mm + 2) for mm in m], np.int32)
    cir, outs = cc.dense_layer(d, W, T)
    cirS, outsS = cc.dense_layer(d, W, None, out_bits=10)
    for _ in range(8):
        x = rng.integers(0, 2, d).astype(np.uint8)
        assert np.array_equal(cc.eval_plain(cir, x, outs), cc.dense_plain(x, W, T))
        bits = cc.eval_plain(cirS, x, outsS).reshape(p, 10)
        assert np.array_equal((bits.astype(np.int64) << np.arange(10)).sum(axis=1), cc.dense_plain(x, W, None))


def test_conv_plain_against_library_correlation():
    c4 = workloads.cfg4(C=3, H=7, Wd=6, O=4)
    x, K, T = c4["x"], c4["K"], c4["T"]
    xs = np.pad(2 * x.astype(np.int64) - 1, ((0, 0), (1, 1), (1, 1)), constant_values=-1)
    for o in range(K.shape[0]):
        dot = correlate(xs, K[o].astype(np.int64), mode="valid")[0]       # sum_c,ky,kx K * x
        S = (dot + K[o].size) // 2                                         # agreements
        for Tt in (T[o], 10, 14, 20):
            want = (S >= Tt).astype(np.uint8)
            got = cc.conv_plain(x, K, np.full(K.shape[0], Tt), 1, 1)[o]
            assert np.array_equal(got, want)


def test_conv_circuit_equals_integer_layer():
    rng = np.random.default_rng(3)
    C_, H, Wd, O = 2, 5, 4, 3
    x = rng.integers(0, 2, (C_, H, Wd)).astype(np.uint8)
    K = (2 * rng.integers(0, 2, (O, C_, 3, 3)) - 1).astype(np.int8)
    T = rng.integers(6, 13, O).astype(np.int32)
    cir, outs = cc.conv_layer(C_, H, Wd, K, T, 1, 1)
    got = cc.eval_plain(cir, x.reshape(-1), outs).reshape(O, H, Wd)
    assert np.array_equal(got, cc.conv_plain(x, K, T, 1, 1))
    # every pixel sums all 18 taps: padding is an (encrypted) zero, not a dropped input
    n_per_pixel = len(cir.gates) / (O * H * Wd)
    one = cc.Circuit(18)
    cc.neuron(one, [(i, 0) for i in range(18)], np.ones(18, np.int8), 9)
    assert abs(n_per_pixel - len(one.gates)) <= 4
    # stride 2, no padding
    cir, outs = cc.conv_layer(C_, H, Wd, K, T, 2, 0)
    got = cc.eval_plain(cir, x.reshape(-1), outs).reshape(O, 2, 1)
    assert np.array_equal(got, cc.conv_plain(x, K, T, 2, 0))


# --------------------------------------------------------------------------- encrypted
def test_small_dense_layer_encrypted_toy(orc, toy_keys):
    rng = np.random.default_rng(11)
    d, p = 9, 4
    W = rng.choice(np.array([-1, 0, 1], np.int8), (p, d))
    T = np.array([0, 3, 2, 20], np.int32)
    x = rng.integers(0, 2, d).astype(np.uint8)
    cir, outs = cc.dense_layer(d, W, T)
    ct = toy_keys.encrypt(x, 3)
    res, wires = cc.eval_encrypted(toy_keys, cir, ct, outs, threads=4)
    assert np.array_equal(toy_keys.decrypt(res), cc.dense_plain(x, W, T))
    res1, _ = cc.eval_encrypted(toy_keys, cir, ct, outs, threads=1)
    assert np.array_equal(res, res1)


def test_one_neuron_encrypted_real_parameters(orc, real_keys):
    rng = np.random.default_rng(12)
    d = 12
    W = (2 * rng.integers(0, 2, (1, d)) - 1).astype(np.int8)
    x = rng.integers(0, 2, d).astype(np.uint8)
    ct = real_keys.encrypt(x, 77)
    for T in (5, 7):
        cir, outs = cc.dense_layer(d, W, np.array([T]))
        res, _ = cc.eval_encrypted(real_keys, cir, ct, outs, threads=8)
        assert real_keys.decrypt(res)[0] == cc.dense_plain(x, W, np.array([T]))[0]


# --------------------------------------------------------------------------- Algorithm 1 as printed
@pytest.mark.parametrize("m", [1, 2, 3, 5, 8, 13, 31, 32])
def test_mux_comparator_all_S_all_T(m):
    w = int(m).bit_length()
    tree = len(popcount_bits(m)[0].gates)
    for T in range(-1, m + 3):
        cir = cc.Circuit(m)
        outs = cc.neuron(cir, [(i, 0) for i in range(m)], np.ones(m, np.int8), T, comparator="mux")
        assert len(cir.gates) == tree + 2 * w              # one MUX (two records) per bit of S
        for S in range(m + 1):
            x = np.zeros(m, np.uint8)
            x[:S] = 1
            assert cc.eval_plain(cir, x, outs)[0] == (1 if S >= T else 0), (m, T, S)


def test_mux_comparator_encrypted_toy(orc, toy_keys):
    rng = np.random.default_rng(21)
    d = 7
    W = (2 * rng.integers(0, 2, (2, d)) - 1).astype(np.int8)
    T = np.array([3, 5], np.int32)
    x = rng.integers(0, 2, d).astype(np.uint8)
    ct = toy_keys.encrypt(x, 4)
    cir, outs = cc.dense_layer(d, W, T, comparator="mux")
    res, _ = cc.eval_encrypted(toy_keys, cir, ct, outs, threads=4)
    assert np.array_equal(toy_keys.decrypt(res), cc.dense_plain(x, W, T))
    folded, fo = cc.dense_layer(d, W, T)
    ref, _ = cc.eval_encrypted(toy_keys, folded, ct, fo, threads=4)
    assert np.array_equal(toy_keys.decrypt(ref), toy_keys.decrypt(res))


# --------------------------------------------------------------------------- the "+1" trick
def test_plus_one_identity_of_the_paper():
    """w.x = (1+w).(1+x) - sum(w) - (1+x).1 and (1+w).(1+x) = 4 * sum of x-bar over w=+1 (Sec. 4.2)."""
    rng = np.random.default_rng(1)
    for _ in range(200):
        d = int(rng.integers(1, 60))
        w = 2 * rng.integers(0, 2, d) - 1
        xb = rng.integers(0, 2, d)
        x = 2 * xb - 1
        assert (w * x).sum() == ((1 + w) * (1 + x)).sum() - w.sum() - (1 + x).sum()
        assert ((1 + w) * (1 + x)).sum() == 4 * xb[w == 1].sum()


@pytest.mark.parametrize("d", [2, 3, 4, 5, 7, 8, 9])
def test_plus_one_unit_exhaustive(d):
    rng = np.random.default_rng(d)
    rows = [np.ones(d, np.int8), -np.ones(d, np.int8)] + [(2 * rng.integers(0, 2, d) - 1).astype(np.int8) for _ in range(4)]
    for w in rows:
        for T in range(-1, d + 3):
            cir, outs = cc.dense_layer(d, w.reshape(1, d), np.array([T]), plus_one=True)
            for bits in itertools.product((0, 1), repeat=d):
                x = np.array(bits, np.uint8)
                assert cc.eval_plain(cir, x, outs)[0] == cc.dense_plain(x, w.reshape(1, d), np.array([T]))[0], (w, T, bits)


@pytest.mark.parametrize("d,p", [(33, 6), (144, 4), (256, 3), (784, 3)])
def test_plus_one_layer_random_and_gate_savings(d, p):
    rng = np.random.default_rng(d)
    W = (2 * rng.integers(0, 2, (p, d)) - 1).astype(np.int8)
    T = rng.integers(d // 3, 2 * d // 3, p).astype(np.int32)
    plain_cir, plain_outs = cc.dense_layer(d, W, T)
    cir, outs = cc.dense_layer(d, W, T, plus_one=True)
    for _ in range(6):
        x = rng.integers(0, 2, d).astype(np.uint8)
        assert np.array_equal(cc.eval_plain(cir, x, outs), cc.dense_plain(x, W, T))
    # per unit about half the gates; the shared popcount of the inputs is paid once per layer
    shared = len(popcount_bits(d)[0].gates)
    per_unit = (len(cir.gates) - shared) / p
    assert per_unit < 0.62 * len(plain_cir.gates) / p
    # a row with a dropped input falls back to the plain unit
    W[0, 0] = 0
    cir2, outs2 = cc.dense_layer(d, W, T, plus_one=True)
    x = rng.integers(0, 2, d).astype(np.uint8)
    assert np.array_equal(cc.eval_plain(cir2, x, outs2), cc.dense_plain(x, W, T))


def test_plus_one_convolution():
    rng = np.random.default_rng(5)
    C_, H, Wd, O = 2, 4, 5, 3
    x = rng.integers(0, 2, (C_, H, Wd)).astype(np.uint8)
    K = (2 * rng.integers(0, 2, (O, C_, 3, 3)) - 1).astype(np.int8)
    T = rng.integers(6, 13, O).astype(np.int32)
    cir, outs = cc.conv_layer(C_, H, Wd, K, T, 1, 1, plus_one=True)
    got = cc.eval_plain(cir, x.reshape(-1), outs).reshape(O, H, Wd)
    assert np.array_equal(got, cc.conv_plain(x, K, T, 1, 1))
    # only 3 channels share each receptive-field popcount here; still fewer gates than the plain units
    assert len(cir.gates) < len(cc.conv_layer(C_, H, Wd, K, T, 1, 1)[0].gates)


def test_plus_one_encrypted_toy(orc, toy_keys):
    rng = np.random.default_rng(23)
    d, p = 6, 3
    W = (2 * rng.integers(0, 2, (p, d)) - 1).astype(np.int8)
    T = np.array([2, 3, 4], np.int32)
    x = rng.integers(0, 2, d).astype(np.uint8)
    ct = toy_keys.encrypt(x, 8)
    cir, outs = cc.dense_layer(d, W, T, plus_one=True)
    res, _ = cc.eval_encrypted(toy_keys, cir, ct, outs, threads=4)
    assert np.array_equal(toy_keys.decrypt(res), cc.dense_plain(x, W, T))


# --------------------------------------------------------------------------- sorting network
def test_swap_sorts_two_bits():
    """SWAP(a, b) = (OR(a, b), AND(a, b)) is (max, min) (Sec. 4.1.1)."""
    for a, b in itertools.product((0, 1), repeat=2):
        assert (a | b, a & b) == (max(a, b), min(a, b))


@pytest.mark.parametrize("m", [1, 2, 3, 4, 5, 6, 7, 8, 9, 11])
def test_sorting_network_unit_exhaustive(m):
    rng = np.random.default_rng(m)
    w = (2 * rng.integers(0, 2, m) - 1).astype(np.int8)
    for T in range(-1, m + 3):
        cir = cc.Circuit(m)
        outs = cc.neuron(cir, [(i, 0) for i in range(m)], w, T, comparator="sort")
        for bits in itertools.product((0, 1), repeat=m):
            x = np.array(bits, np.uint8)
            assert cc.eval_plain(cir, x, outs)[0] == cc.dense_plain(x, w.reshape(1, m), np.array([T]))[0]


@pytest.mark.parametrize("m", [16, 33, 100, 144, 256])
def test_sorting_network_unit_random_and_size(m):
    rng = np.random.default_rng(m)
    w = rng.choice(np.array([-1, 0, 1], np.int8), m, p=[0.45, 0.1, 0.45])
    live = int((w != 0).sum())
    n = 1 << (live - 1).bit_length()
    full = 2 * (n // 4) * n.bit_length() * (n.bit_length() - 1)      # 2 gates x (n/4) log n (log n + 1) swaps
    for T in (1, live // 3, live // 2, live):
        cir = cc.Circuit(m)
        outs = cc.neuron(cir, [(i, 0) for i in range(m)], w, T, comparator="sort")
        assert len(cir.gates) <= full
        for _ in range(5):
            x = rng.integers(0, 2, m).astype(np.uint8)
            assert cc.eval_plain(cir, x, outs)[0] == cc.dense_plain(x, w.reshape(1, m), np.array([T]))[0]
