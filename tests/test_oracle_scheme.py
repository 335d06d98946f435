"""Pins for the oracle's scheme layer: keys, encryption, the steps of a bootstrapped
gate and the gate itself.

With noise-free keys (noise_log2 <= -40 makes the integer sampler return 0) several
steps have closed forms that the brute-force product definition can evaluate; the
whole gate is pinned by its truth table after decryption and by the predicted
variance of its output noise.
"""
import itertools

import numpy as np
import pytest

M32 = (1 << 32) - 1
MU = 1 << 29
TRUTH = {"NAND": lambda a, b: 1 - (a & b), "AND": lambda a, b: a & b, "OR": lambda a, b: a | b,
         "NOR": lambda a, b: 1 - (a | b), "XOR": lambda a, b: a ^ b, "XNOR": lambda a, b: 1 - (a ^ b)}


def s32(x):
    x = np.asarray(x, dtype=np.int64) & M32
    return np.where(x >= 1 << 31, x - (1 << 32), x)


def rnd_u32(rng, n):
    return rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32)


@pytest.fixture(scope="module")
def quiet_keys(orc):
    """Toy ring, no noise anywhere."""
    return orc.Keys(orc.Params(12, 32, 1, 2, 10, 8, 2, -60, -60), 777)


# --------------------------------------------------------------------------- keys, enc/dec
def test_key_bits_and_sizes(orc, real_keys):
    K = real_keys
    assert set(np.unique(K.lwe_sk)) <= {0, 1} and set(np.unique(K.trlwe_sk)) <= {0, 1}
    assert 200 < K.lwe_sk.sum() < 300 and 450 < K.trlwe_sk.sum() < 574
    assert K.bk.size == 500 * 4 * 2 * 1024            # 16.4 MB
    assert K.ksk.size == 1024 * 8 * 3 * 501           # 49.2 MB


def test_fresh_ciphertext_phase(orc, real_keys):
    bits = np.random.default_rng(0).integers(0, 2, 4000).astype(np.uint8)
    ct = real_keys.encrypt(bits, 31337)
    assert np.array_equal(real_keys.decrypt(ct), bits)
    err = s32(real_keys.phase(ct).astype(np.int64) - np.where(bits, MU, -MU))
    assert abs(err.std() / 2.0**17 - 1) < 0.05 and abs(err.mean()) < 2.0**17 / 10
    # the mask words are the ENC_A stream, sample k word j at index k*n + j
    assert ct[3, 5] == orc.rand(31337, "ENC_A", 3 * 500 + 5) >> 32
    # noiseless trivial samples
    assert real_keys.phase(real_keys.trivial(1))[0] == MU
    assert real_keys.phase(real_keys.trivial(0))[0] == (-MU) & M32


def test_bootstrapping_key_rows_encrypt_gadget_times_key_bit(orc, toy_keys):
    """phase(row(u,j)) = s_i * 2^(32-10(j+1)) * (u ? 1 : -S) + small noise."""
    K, P = toy_keys, toy_keys.P
    N = P.N
    for i in range(P.n):
        rows = K.bk_row(i).reshape(2 * P.bk_l, 2, N)
        for r in range(2 * P.bk_l):
            u, j = divmod(r, P.bk_l)
            ph = s32(rows[r, 1].astype(np.int64) - orc.negacyclic(rows[r, 0], K.trlwe_sk, "definition"))
            g = int(K.lwe_sk[i]) << (32 - P.bk_Bgbit * (j + 1))
            want = np.zeros(N, np.int64)
            if u == 1:
                want[0] = g
            else:
                want = -g * K.trlwe_sk.astype(np.int64)
            err = s32(ph - want)
            assert np.abs(err).max() <= 6 * 128 + 1            # noise stdev 2^-25 = 128 units


def test_key_switching_key_rows(orc, real_keys):
    K, P = real_keys, real_keys.P
    rows = K.ksk.reshape(P.N, P.ks_t, 3, P.n + 1)
    rng = np.random.default_rng(2)
    for _ in range(300):
        i, j, v = rng.integers(0, P.N), rng.integers(0, P.ks_t), rng.integers(1, 4)
        ph = int(K.phase(rows[i, j, v - 1])[0])
        want = (int(v) * int(K.trlwe_sk[i])) << (32 - 2 * (j + 1))
        assert abs(int(s32(ph - want))) <= 6 * 2**17 + 1


# --------------------------------------------------------------------------- steps, sigma = 0
def gadget_round(K, x):
    """sum_j d_j 2^(32 - Bgbit (j+1)) for each word of x."""
    P = K.P
    out = np.zeros(len(x), np.int64)
    for m, v in enumerate(x):
        d = K.decompose(int(v))
        out[m] = sum(int(d[j]) << (32 - P.bk_Bgbit * (j + 1)) for j in range(P.bk_l))
    return out


def test_external_product_phase_closed_form(orc, quiet_keys):
    """No noise: phase(BK_i [.] D) = s_i * (round(D_B) - S * round(D_A))."""
    K, N = quiet_keys, quiet_keys.P.N
    rng = np.random.default_rng(4)
    for i in range(K.P.n):
        D = rnd_u32(rng, 2 * N)
        out = K.external_product(i, D)
        rA = (gadget_round(K, D[:N]) & M32).astype(np.uint32)
        rB = gadget_round(K, D[N:])
        want = int(K.lwe_sk[i]) * (rB - orc.negacyclic(rA, K.trlwe_sk, "definition").astype(np.int64))
        assert np.array_equal(K.trlwe_phase(out), (want & M32).astype(np.uint32))


def test_first_rotation_step_is_exact(orc, quiet_keys):
    """ACC = (0, X^-b v) has coefficients on the gadget grid, so with noise-free keys the
    first step gives phase = X^(s_0 a_0) * phase exactly."""
    K, P = quiet_keys, quiet_keys.P
    N = P.N
    for bbar, a0 in itertools.product([0, 5, N + 3], [1, 7, N, 2 * N - 1]):
        acc = K.acc_init(bbar)
        bar = np.zeros(P.n + 1, np.uint32)
        bar[0] = a0
        bar[P.n] = bbar
        out = K.blind_rotate(bar, acc)
        want = orc.mul_by_xpow(acc[N:], a0 if K.lwe_sk[0] else 0)
        assert np.array_equal(K.trlwe_phase(out), want)


def test_blind_rotation_rotates_by_the_phase(orc, quiet_keys):
    """No noise: the accumulator's phase is X^(sum s_i a_i - b) * v up to gadget rounding."""
    K, P = quiet_keys, quiet_keys.P
    N = P.N
    rng = np.random.default_rng(6)
    for _ in range(10):
        bar = rng.integers(0, 2 * N, P.n + 1).astype(np.uint32)
        acc = K.blind_rotate(bar, K.acc_init(bar[P.n]))
        rot = (int((bar[:P.n] * K.lwe_sk).sum()) - int(bar[P.n])) % (2 * N)
        want = orc.mul_by_xpow(np.full(N, MU, np.uint32), rot)
        err = s32(K.trlwe_phase(acc).astype(np.int64) - want)
        assert np.abs(err).max() < P.n * (N + 1) * 2**11


def test_sample_extract_is_constant_coefficient(orc, toy_keys):
    """phase_S(extract(acc)) equals coefficient 0 of the TRLWE phase."""
    K, N = toy_keys, toy_keys.P.N
    rng = np.random.default_rng(8)
    acc = rnd_u32(rng, 2 * N)
    ext = K.sample_extract(acc)
    ph = (int(ext[N]) - int((ext[:N].astype(np.int64) * K.trlwe_sk).sum())) & M32
    assert ph == int(K.trlwe_phase(acc)[0])
    assert ext[0] == acc[0] and ext[1] == (-int(acc[N - 1])) & M32 and ext[N] == acc[N]


def test_key_switch_phase_closed_form(orc):
    """No noise: phase_s(out) = phase_S(in) - sum_i S_i * (round16(a_i) - a_i)."""
    K = orc.Keys(orc.Params(20, 64, 1, 2, 10, 8, 2, -60, -60), 99)
    N = K.P.N
    rng = np.random.default_rng(10)
    for _ in range(20):
        ext = rnd_u32(rng, N + 1)
        out = K.key_switch(ext)
        a = ext[:N].astype(np.int64)
        rounded = ((a + (1 << 15)) & M32) & ~0xFFFF
        ph_in = int(ext[N]) - int((a * K.trlwe_sk).sum())
        want = (ph_in - int(((rounded - a) * K.trlwe_sk).sum())) & M32
        assert int(K.phase(out)[0]) == want


def test_key_switch_noise_bound(orc, real_keys):
    K, N = real_keys, real_keys.P.N
    rng = np.random.default_rng(12)
    errs = []
    for _ in range(40):
        ext = rnd_u32(rng, N + 1)
        ph_in = (int(ext[N]) - int((ext[:N].astype(np.int64) * K.trlwe_sk).sum())) & M32
        errs.append(int(s32(int(K.phase(K.key_switch(ext))[0]) - ph_in)))
    # predicted stdev: sqrt(N t (3/4)) 2^17 + rounding ~ 2^-8.7 => 1.0e7 units
    assert 0.6e7 < np.std(errs) < 1.6e7


# --------------------------------------------------------------------------- whole gate
def test_precombination_constants(orc, toy_keys):
    """Each gate's affine map sends the four input phase pairs to +-1/8, +-3/8 (AND family) or
    +-1/4 (XOR family) with the sign of its truth table (noise-free trivial samples)."""
    K = toy_keys
    t = {0: K.trivial(0), 1: K.trivial(1)}
    for op, f in TRUTH.items():
        for a, b, na, nb in itertools.product((0, 1), repeat=4):
            ph = int(s32(K.phase(K.precombine(op, t[a], t[b], na, nb))[0]))
            want = f(a ^ na, b ^ nb)
            assert abs(ph) in ((MU, 3 * MU) if op not in ('XOR', 'XNOR') else (2 * MU,)) and (ph > 0) == bool(want), (op, a, b, na, nb, ph)


@pytest.mark.parametrize("method", [0, 1, 2])
def test_toy_gate_truth_tables_any_product(orc, toy_keys, method):
    K = toy_keys
    ct = K.encrypt(np.array([0, 1], np.uint8), 5)
    orc.lib().orc_set_product_method(method)
    try:
        for op, f in TRUTH.items():
            for a, b in itertools.product((0, 1), repeat=2):
                assert K.decrypt(K.gate(op, ct[a], ct[b]))[0] == f(a, b)
    finally:
        orc.lib().orc_set_product_method(0)


def test_gate_bytes_do_not_depend_on_product_method(orc, toy_keys):
    K = toy_keys
    ct = K.encrypt(np.array([0, 1, 1], np.uint8), 6)
    outs = []
    for method in (0, 1, 2):
        orc.lib().orc_set_product_method(method)
        outs.append([K.gate(op, ct[0], ct[1], 0, 1) for op in TRUTH])
    orc.lib().orc_set_product_method(0)
    for o in outs[1:]:
        assert all(np.array_equal(x, y) for x, y in zip(o, outs[0]))


def test_real_parameter_truth_tables_and_noise(orc, real_keys):
    """All six gates on all input pairs, with and without negated inputs, at n=500 N=1024;
    output noise variance against the prediction
      n * 2l * N * (Bg^2/12) * sigma_bk^2  +  N t (3/4) sigma_ks^2   (stdev ~ 2^-6.3)."""
    K = real_keys
    rng = np.random.default_rng(14)
    bits = rng.integers(0, 2, 64).astype(np.uint8)
    ct = K.encrypt(bits, 2024)
    n1 = K.P.n + 1
    recs, want = [], []
    nw = len(bits)
    for op, f in TRUTH.items():
        for a, b in itertools.product((0, 1), repeat=2):
            for na, nb in ((0, 0), (1, 0), (0, 1), (1, 1)):
                i0 = int(np.nonzero(bits == a)[0][rng.integers(0, (bits == a).sum())])
                i1 = int(np.nonzero(bits == b)[0][rng.integers(0, (bits == b).sum())])
                recs.append((orc.OP[op], na, nb, 0, i0, i1, nw + len(recs)))
                want.append(f(a ^ na, b ^ nb))
    gates = np.array(recs, dtype=orc.GATE_DTYPE)
    wires = np.zeros((nw + len(recs), n1), np.uint32)
    wires[:nw] = ct
    K.gate_batch(gates, wires, threads=8)
    out = wires[nw:]
    assert np.array_equal(K.decrypt(out), np.array(want, np.uint8))
    err = s32(K.phase(out).astype(np.int64) - np.where(np.array(want) > 0, MU, -MU)) / 2.0**32
    pred = 500 * 4 * 1024 * (1024**2 / 12) * 2.0**-50 + 1024 * 8 * 0.75 * 2.0**-30
    assert 0.65 * pred < err.var() < 1.4 * pred, (err.var(), pred)
    # threads do not change bytes: redo a few single-threaded through the scalar entry point
    for k in (0, 17, 95):
        g = gates[k]
        assert np.array_equal(K.gate(int(g["op"]), ct[g["in0"]], ct[g["in1"]], int(g["neg0"]), int(g["neg1"])),
                              out[k])


# --------------------------------------------------------------------------- multiplexer
def test_mux_truth_table_toy_and_real(orc, toy_keys, real_keys):
    """MUX(s, a, b) = a if s else b (Sec. 4.1) for all eight inputs and negation flags."""
    for K, flags in ((toy_keys, list(itertools.product((0, 1), repeat=3))), (real_keys, [(0, 0, 0), (1, 0, 1)])):
        ct = K.encrypt(np.array([0, 1], np.uint8), 17)
        for s, a, b in itertools.product((0, 1), repeat=3):
            for ns, na, nb in flags:
                got = K.decrypt(K.mux(ct[s], ct[a], ct[b], ns, na, nb))[0]
                assert got == ((a ^ na) if (s ^ ns) else (b ^ nb)), (s, a, b, ns, na, nb)


def test_mux_is_two_bootstraps_summed_then_switched(orc, toy_keys):
    """phase_S(u1 + u2 + 1/8) is +-1/8 with the sign of the selected input, where u1, u2 are the
    ring-key samples of AND(s, a) and AND(NOT s, b); MUX key-switches exactly that sum."""
    K, N = toy_keys, toy_keys.P.N
    ct = K.encrypt(np.array([0, 1], np.uint8), 18)
    for s, a, b in itertools.product((0, 1), repeat=3):
        u1 = K.bootstrap_extract(K.precombine("AND", ct[s], ct[a]))
        u2 = K.bootstrap_extract(K.precombine("AND", ct[s], ct[b], 1, 0))
        u = (u1 + u2).astype(np.uint32)
        u[N] = (int(u[N]) + MU) & M32
        ph = int(s32((int(u[N]) - int((u[:N].astype(np.int64) * K.trlwe_sk).sum())) & M32))
        want = a if s else b
        assert abs(abs(ph) - MU) < MU // 4 and (ph > 0) == bool(want)
        assert np.array_equal(K.key_switch(u), K.mux(ct[s], ct[a], ct[b]))


def test_mux_batch_records_match_scalar_entry_point(orc, toy_keys):
    K = toy_keys
    bits = np.array([0, 1, 1, 0], np.uint8)
    ct = K.encrypt(bits, 19)
    n1 = K.P.n + 1
    wires = np.zeros((8, n1), np.uint32)
    wires[:4] = ct
    recs = np.array([(orc.OP["MUX"], 0, 0, 0, 1, 2, 4), (orc.OP["MUX_ELSE"], 0, 1, 0, 1, 3, 4),
                     (orc.OP["AND"], 0, 0, 0, 1, 2, 5),
                     (orc.OP["MUX"], 1, 0, 0, 0, 3, 6), (orc.OP["MUX_ELSE"], 1, 0, 0, 0, 1, 6)], dtype=orc.GATE_DTYPE)
    K.gate_batch(recs, wires, threads=3)
    assert np.array_equal(wires[4], K.mux(ct[1], ct[2], ct[3], 0, 0, 1))
    assert np.array_equal(wires[5], K.gate("AND", ct[1], ct[2]))
    assert np.array_equal(wires[6], K.mux(ct[0], ct[3], ct[1], 1, 0, 0))
    with pytest.raises(ValueError):                      # a lone first half is malformed
        K.gate_batch(recs[:1], wires, threads=1)
