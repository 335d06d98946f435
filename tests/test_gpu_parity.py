"""GPU parity: ciphertext bytes produced by the HIP library (through its C ABI) against the CPU
oracle, on the same seeded keys and inputs.  All arithmetic is exact modulo 2^32, so the bar is
bit-for-bit equality; decrypted bits are also checked against plain truth tables / integer layers.
"""
import itertools
import os
import sys

import numpy as np
import pytest

import workloads
from oracle import circuits as cc

pytestmark = pytest.mark.gpu

TRUTH = {"NAND": lambda a, b: 1 - (a & b), "AND": lambda a, b: a & b, "OR": lambda a, b: a | b,
         "NOR": lambda a, b: 1 - (a | b), "XOR": lambda a, b: a ^ b, "XNOR": lambda a, b: 1 - (a ^ b)}
OPNAMES = ["NAND", "AND", "OR", "NOR", "XOR", "XNOR"]


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1806_03461_amd as T
    sk, ck = T.tfhe_keygen(T.default_params(), workloads.KEY_SEED)
    T.tfhe_cloud_key_upload(ck)
    return T, sk, ck


def run_batch(T, ck, op, cta, ctb):
    import torch
    a, b = T.to_device(cta), T.to_device(ctb)
    out = torch.empty_like(a)
    T.tfhe_gate_batch(ck, op, a, b, out, a.shape[0])
    torch.cuda.synchronize()
    return T.to_host(out)


def oracle_batch(keys, op, cta, ctb, threads=16):
    n1 = cta.shape[1]
    cnt = cta.shape[0]
    wires = np.zeros((3 * cnt, n1), np.uint32)
    wires[:cnt], wires[cnt:2 * cnt] = cta, ctb
    recs = np.array([(cc.OP[op], 0, 0, 0, i, cnt + i, 2 * cnt + i) for i in range(cnt)], dtype=cc.GATE_DTYPE)
    keys.gate_batch(recs, wires, threads)
    return wires[2 * cnt:]


def test_cfg1_sixteen_gates_bit_exact(gpu, real_keys):
    T, sk, ck = gpu
    c = workloads.cfg1()
    cta = T.tfhe_encrypt(sk, c["enc_seed"], c["a"])
    ctb = T.tfhe_encrypt(sk, c["enc_seed"] + 1, c["b"])
    assert np.array_equal(cta, real_keys.encrypt(c["a"], c["enc_seed"]))
    got = np.concatenate([run_batch(T, ck, "NAND", cta[:8], ctb[:8]), run_batch(T, ck, "XNOR", cta[8:], ctb[8:])])
    want = np.concatenate([oracle_batch(real_keys, "NAND", cta[:8], ctb[:8]),
                           oracle_batch(real_keys, "XNOR", cta[8:], ctb[8:])])
    assert np.array_equal(got, want)
    bits = T.tfhe_decrypt(sk, got)
    plain = [TRUTH[o](int(a), int(b)) for o, a, b in zip(c["ops"], c["a"], c["b"])]
    assert list(bits) == plain


@pytest.mark.parametrize("op", OPNAMES)
def test_every_gate_kind_ragged_batch(gpu, real_keys, op):
    """7 gates: not a multiple of any gates-per-workgroup setting; covers all four input pairs."""
    T, sk, ck = gpu
    a = np.array([0, 0, 1, 1, 1, 0, 1], np.uint8)
    b = np.array([0, 1, 0, 1, 1, 0, 0], np.uint8)
    cta, ctb = T.tfhe_encrypt(sk, 11, a), T.tfhe_encrypt(sk, 12, b)
    got = run_batch(T, ck, op, cta, ctb)
    assert np.array_equal(got, oracle_batch(real_keys, op, cta, ctb))
    assert list(T.tfhe_decrypt(sk, got)) == [TRUTH[op](int(x), int(y)) for x, y in zip(a, b)]


def test_rotation_amounts_at_every_boundary(gpu, real_keys):
    """Inputs built word by word (not encryptions) so that the rotation amounts a-bar of the 500
    blind-rotation steps sit on the values where the rotated read changes shape: 0 (no rotation),
    multiples of 64 (a lane-aligned wrap), one off them, N - 1, N, N + 1 (the sign change of
    X^N = -1), 2N - 1, and the two ties of the rounding to 2N levels.  The oracle takes any words;
    the bar is equal bytes.  (Sec. 3.2: the gate bootstrapping under every BNN gate.)"""
    T, sk, ck = gpu
    n = 500
    special = [0, 1, 2, 31, 32, 63, 64, 65, 127, 128, 129, 511, 512, 513, 959, 960, 961, 1023, 1024, 1025,
               1087, 1088, 1089, 1535, 1536, 1984, 2046, 2047]
    rows = []
    for v in special:                                   # the same amount in every step
        rows.append(np.full(n + 1, v << 21, np.uint64))
    for g in range(12):                                 # the amounts in turn, from a different start per gate
        rows.append(np.array([special[(j * (g + 1) + g) % len(special)] << 21 for j in range(n + 1)], np.uint64))
    for g, tie in enumerate([(1 << 20), (1 << 20) - 1, -(1 << 20), -(1 << 20) - 1]):   # on and beside a tie
        rows.append(np.array([(special[(j + g) % len(special)] << 21) + tie for j in range(n + 1)], np.int64).astype(np.uint64))
    cta = (np.stack(rows) & 0xFFFFFFFF).astype(np.uint32)
    ctb = np.zeros_like(cta)
    for op in ("OR", "NAND"):                           # multiplier +1 and -1 in front of the sum
        got = run_batch(T, ck, op, cta, ctb)
        assert np.array_equal(got, oracle_batch(real_keys, op, cta, ctb)), op


def test_empty_and_in_place_batches(gpu, real_keys):
    import torch
    T, sk, ck = gpu
    T.tfhe_gate_batch(ck, "AND", 0, 0, 0, 0)                       # count 0: no-op, pointers unused
    a = np.array([1, 0, 1], np.uint8)
    cta, ctb = T.tfhe_encrypt(sk, 21, a), T.tfhe_encrypt(sk, 22, a[::-1].copy())
    da, db = T.to_device(cta), T.to_device(ctb)
    T.tfhe_gate_batch(ck, "OR", da, db, da, 3)                     # out aliases a
    torch.cuda.synchronize()
    assert np.array_equal(T.to_host(da), oracle_batch(real_keys, "OR", cta, ctb))


def test_mixed_gate_stream_with_negated_inputs(gpu, real_keys):
    """A small layer through bnn_dense_lower + tfhe_gate_stream: every wire equals the oracle's
    evaluation of the same records, and the oracle's own lowering gives the same output bytes."""
    import torch
    T, sk, ck = gpu
    rng = np.random.default_rng(5)
    d, p = 14, 3
    W = rng.choice(np.array([-1, 0, 1], np.int8), (p, d), p=[0.45, 0.1, 0.45])
    Tt = np.array([4, 7, 6], np.int32)
    x = rng.integers(0, 2, d).astype(np.uint8)
    ctx = T.tfhe_encrypt(sk, 31, x)
    gates, outs, nw = T.bnn_dense_lower(d, W, Tt, p)
    wires = np.zeros((nw, 501), np.uint32)
    wires[:d] = ctx
    wires[d], wires[d + 1] = T.tfhe_trivial(T.default_params(), 0), T.tfhe_trivial(T.default_params(), 1)
    dev = T.to_device(wires)
    T.tfhe_gate_stream(ck, gates, dev, nw)
    torch.cuda.synchronize()
    got = T.to_host(dev)
    want = wires.copy()
    real_keys.run_gates(gates, want, threads=16)
    assert np.array_equal(got, want)
    # the layer entry point, against the oracle's independent circuit builder
    out = torch.empty((p, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted(ck, T.to_device(ctx), d, W, Tt, p, out)
    torch.cuda.synchronize()
    cir, o = cc.dense_layer(d, W, Tt)
    ref, _ = cc.eval_encrypted(real_keys, cir, ctx, o, threads=16)
    assert np.array_equal(T.to_host(out), ref)
    assert np.array_equal(T.tfhe_decrypt(sk, T.to_host(out)), cc.dense_plain(x, W, Tt))


def test_large_batch_truth_tables_and_sampled_parity(gpu, real_keys):
    """4099 gates (several workgroups per CU plus a ragged tail): all outputs decrypt to the truth
    table; 24 sampled outputs are compared byte for byte with the oracle."""
    T, sk, ck = gpu
    rng = np.random.default_rng(7)
    cnt = 4099
    a, b = rng.integers(0, 2, cnt).astype(np.uint8), rng.integers(0, 2, cnt).astype(np.uint8)
    cta, ctb = T.tfhe_encrypt(sk, 41, a), T.tfhe_encrypt(sk, 42, b)
    for op in ("NAND", "XOR"):
        got = run_batch(T, ck, op, cta, ctb)
        assert np.array_equal(T.tfhe_decrypt(sk, got), np.array([TRUTH[op](int(x), int(y)) for x, y in zip(a, b)], np.uint8))
        idx = np.concatenate([rng.integers(0, cnt, 20), [0, 1, cnt - 2, cnt - 1]])
        assert np.array_equal(got[idx], oracle_batch(real_keys, op, cta[idx], ctb[idx]))


def test_rounding_margin_of_the_split_integer_products(gpu):
    """The transform-domain products are rounded to integers; the distance of the raw values from
    an integer must stay far below 1/2 for the rounding to be exact."""
    T, sk, ck = gpu
    rng = np.random.default_rng(9)
    a = rng.integers(0, 2, 64).astype(np.uint8)
    cta, ctb = T.tfhe_encrypt(sk, 51, a), T.tfhe_encrypt(sk, 52, a[::-1].copy())
    T.tfhe_rounding_margin_enable(ck, True)
    try:
        run_batch(T, ck, "XNOR", cta, ctb)
        worst = T.tfhe_rounding_margin_read(ck)
    finally:
        T.tfhe_rounding_margin_enable(ck, False)
    assert 0 < worst < 1e-3, worst


def test_bad_gate_records_are_rejected(gpu):
    import torch
    T, sk, ck = gpu
    wires = torch.zeros((4, 501), dtype=torch.int32, device="cuda")
    def rec(op, i0, i1, out):
        return np.array([(op, 0, 0, 0, i0, i1, out)], dtype=T.GATE_DTYPE)
    for bad in (rec(9, 0, 1, 2), rec(1, 0, 7, 2), rec(1, 0, 1, -1),
                np.concatenate([rec(1, 0, 1, 2), rec(1, 0, 1, 2)]),       # wire written twice
                np.concatenate([rec(1, 3, 1, 2), rec(1, 0, 1, 3)])):      # reads a later record's output
        with pytest.raises(T.TfheError):
            T.tfhe_gate_stream(ck, bad, wires, 4)


def test_other_parameter_set_general_key_switch(real_keys):
    """n=300, Bgbit=8, key switch with 5 base-8 digits: exercises the one-gate-per-workgroup key
    switch and the run-time gadget base, against an oracle key set of the same parameters."""
    import torch
    import paper_1806_03461_amd as T
    from oracle import oracle as orc
    P = T.Params(300, 1024, 1, 2, 8, 5, 3, -15, -25)
    sk, ck = T.tfhe_keygen(P, 777)
    keys = orc.Keys(orc.Params(300, 1024, 1, 2, 8, 5, 3, -15, -25), 777)
    assert np.array_equal(T.tfhe_export_key(ck, T.KEY_KSK_RAW), keys.ksk)
    a = np.array([0, 1, 1, 0, 1], np.uint8)
    b = np.array([1, 1, 0, 0, 1], np.uint8)
    cta, ctb = T.tfhe_encrypt(sk, 5, a), T.tfhe_encrypt(sk, 6, b)
    for op in ("AND", "XNOR"):
        da, db = T.to_device(cta), T.to_device(ctb)
        out = torch.empty_like(da)
        T.tfhe_gate_batch(ck, op, da, db, out, 5)
        torch.cuda.synchronize()
        got = T.to_host(out)
        want = np.stack([keys.gate(op, cta[i], ctb[i]) for i in range(5)])
        assert np.array_equal(got, want)
        assert list(T.tfhe_decrypt(sk, got)) == [TRUTH[op](int(x), int(y)) for x, y in zip(a, b)]


def test_results_do_not_depend_on_batching(gpu):
    """The same gates evaluated twice, in another order, and as a gate stream split over several
    depths give identical bytes: no result depends on which workgroup or launch computed it."""
    import torch
    T, sk, ck = gpu
    rng = np.random.default_rng(13)
    cnt = 300
    a, b = rng.integers(0, 2, cnt).astype(np.uint8), rng.integers(0, 2, cnt).astype(np.uint8)
    cta, ctb = T.tfhe_encrypt(sk, 81, a), T.tfhe_encrypt(sk, 82, b)
    first = run_batch(T, ck, "AND", cta, ctb)
    assert np.array_equal(first, run_batch(T, ck, "AND", cta, ctb))
    perm = rng.permutation(cnt)
    assert np.array_equal(first[perm], run_batch(T, ck, "AND", cta[perm], ctb[perm]))
    # as a stream: wires = [a | b | out], records in reverse order
    wires = torch.zeros((3 * cnt, 501), dtype=torch.int32, device="cuda")
    wires[:cnt], wires[cnt:2 * cnt] = T.to_device(cta), T.to_device(ctb)
    recs = np.array([(T.AND, 0, 0, 0, i, cnt + i, 2 * cnt + i) for i in reversed(range(cnt))], dtype=T.GATE_DTYPE)
    T.tfhe_profile_enable(ck, True)
    T.tfhe_profile_read(ck, reset=True)
    T.tfhe_gate_stream(ck, recs, wires, 3 * cnt)
    torch.cuda.synchronize()
    prof = T.tfhe_profile_read(ck, reset=True)
    T.tfhe_profile_enable(ck, False)
    assert np.array_equal(T.to_host(wires[2 * cnt:]), first)
    assert prof["gates"] == cnt and prof["blind_rotate_launches"] == 1 and prof["blind_rotate_ms"] > 0


def test_mux_gate_batch_and_stream(gpu, real_keys):
    """The three-input multiplexer: all eight input combinations (plus a ragged tail) through
    tfhe_mux_batch, and a small layer whose comparator is Algorithm 1's MUX chain, byte for byte
    against the oracle."""
    import torch
    T, sk, ck = gpu
    s = np.array([0, 0, 0, 0, 1, 1, 1, 1, 1, 0, 1], np.uint8)
    a = np.array([0, 0, 1, 1, 0, 0, 1, 1, 0, 1, 1], np.uint8)
    b = np.array([0, 1, 0, 1, 0, 1, 0, 1, 1, 0, 0], np.uint8)
    cs, ca, cb = T.tfhe_encrypt(sk, 91, s), T.tfhe_encrypt(sk, 92, a), T.tfhe_encrypt(sk, 93, b)
    out = torch.empty((len(s), 501), dtype=torch.int32, device="cuda")
    T.tfhe_mux_batch(ck, T.to_device(cs), T.to_device(ca), T.to_device(cb), out, len(s))
    torch.cuda.synchronize()
    got = T.to_host(out)
    assert list(T.tfhe_decrypt(sk, got)) == [int(x if c else y) for c, x, y in zip(s, a, b)]
    want = np.stack([real_keys.mux(cs[i], ca[i], cb[i]) for i in range(len(s))])
    assert np.array_equal(got, want)
    # Algorithm 1 as printed, inside a layer
    rng = np.random.default_rng(95)
    d, p = 11, 3
    W = rng.choice(np.array([-1, 0, 1], np.int8), (p, d), p=[0.45, 0.1, 0.45])
    Tt = np.array([3, 6, 5], np.int32)
    x = rng.integers(0, 2, d).astype(np.uint8)
    ctx = T.tfhe_encrypt(sk, 96, x)
    res = torch.empty((p, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted_opts(ck, T.to_device(ctx), d, W, Tt, p, res, 0, T.LOWER_MUX_COMPARATOR)
    torch.cuda.synchronize()
    cir, o = cc.dense_layer(d, W, Tt, comparator="mux")
    ref, _ = cc.eval_encrypted(real_keys, cir, ctx, o, threads=16)
    assert np.array_equal(T.to_host(res), ref)
    assert np.array_equal(T.tfhe_decrypt(sk, T.to_host(res)), cc.dense_plain(x, W, Tt))
    # malformed pairs are refused
    wires = torch.zeros((6, 501), dtype=torch.int32, device="cuda")
    lone = np.array([(T.MUX, 0, 0, 0, 0, 1, 4)], dtype=T.GATE_DTYPE)
    other_sel = np.array([(T.MUX, 0, 0, 0, 0, 1, 4), (T.MUX_ELSE, 0, 0, 0, 2, 3, 4)], dtype=T.GATE_DTYPE)
    for bad in (lone, other_sel, other_sel[1:]):
        with pytest.raises(T.TfheError):
            T.tfhe_gate_stream(ck, bad, wires, 6)


def test_matrix_core_key_switch(gpu, real_keys):
    """The int8 matrix-core key switch on batches wide enough for whole workgroups: a ragged
    batch (two full 256-gate workgroups and a tail) whole against the oracle, a multiplexer batch
    (every second launch item writes nothing), and a gate stream whose records carry scattered
    output wires and multiplexer pairs."""
    import torch
    T, sk, ck = gpu
    rng = np.random.default_rng(23)
    cnt = 700
    a, b, s = (rng.integers(0, 2, cnt).astype(np.uint8) for _ in range(3))
    cta, ctb, cts = T.tfhe_encrypt(sk, 101, a), T.tfhe_encrypt(sk, 102, b), T.tfhe_encrypt(sk, 103, s)
    got = run_batch(T, ck, "OR", cta, ctb)
    assert np.array_equal(got, oracle_batch(real_keys, "OR", cta, ctb))
    # 300 multiplexers = 600 launch items
    m = 300
    out = torch.empty((m, 501), dtype=torch.int32, device="cuda")
    T.tfhe_mux_batch(ck, T.to_device(cts[:m]), T.to_device(cta[:m]), T.to_device(ctb[:m]), out, m)
    torch.cuda.synchronize()
    got = T.to_host(out)
    assert np.array_equal(T.tfhe_decrypt(sk, got), np.where(s[:m] == 1, a[:m], b[:m]))
    for i in list(rng.integers(0, m, 12)) + [0, m - 1]:
        assert np.array_equal(got[i], real_keys.mux(cts[i], cta[i], ctb[i])), i
    # a layer of 200 small units with Algorithm 1's comparator: every level holds 600+ items, MUX pairs included
    d, p = 6, 200
    W = (2 * rng.integers(0, 2, (p, d)) - 1).astype(np.int8)
    Tt = rng.integers(1, 6, p).astype(np.int32)
    x = rng.integers(0, 2, d).astype(np.uint8)
    ctx = T.tfhe_encrypt(sk, 104, x)
    res = torch.empty((p, 501), dtype=torch.int32, device="cuda")
    T.tfhe_profile_enable(ck, True)
    T.tfhe_profile_read(ck, reset=True)
    T.bnn_dense_encrypted_opts(ck, T.to_device(ctx), d, W, Tt, p, res, 0, T.LOWER_MUX_COMPARATOR)
    torch.cuda.synchronize()
    prof = T.tfhe_profile_read(ck, reset=True)
    T.tfhe_profile_enable(ck, False)
    assert prof["gates"] / prof["key_switch_launches"] >= 512
    host = T.to_host(res)
    assert np.array_equal(T.tfhe_decrypt(sk, host), cc.dense_plain(x, W, Tt))
    for j in (0, 57, 199):
        cir, o = cc.dense_layer(d, W[j:j + 1], Tt[j:j + 1], comparator="mux")
        ref, _ = cc.eval_encrypted(real_keys, cir, ctx, o, threads=16)
        assert np.array_equal(host[j], ref[0]), j


def test_imported_cloud_key_serves_gates(gpu, real_keys):
    """A server that was handed only raw cloud-key material (here: the oracle's own arrays, no
    secret key involved) evaluates gates to the oracle's bytes."""
    T, sk, ck = gpu
    _, served = T.tfhe_import_keys(T.default_params(), bk_raw=real_keys.bk, ksk_raw=real_keys.ksk)
    rng = np.random.default_rng(31)
    a, b = rng.integers(0, 2, 9).astype(np.uint8), rng.integers(0, 2, 9).astype(np.uint8)
    cta, ctb = real_keys.encrypt(a, 111), real_keys.encrypt(b, 112)
    got = run_batch(T, served, "NOR", cta, ctb)
    assert np.array_equal(got, oracle_batch(real_keys, "NOR", cta, ctb))
    assert list(T.tfhe_decrypt(sk, got)) == [int(not (x or y)) for x, y in zip(a, b)]


_CHUNK_SCRIPT = r"""
import hashlib, sys
import numpy as np, torch
sys.path.insert(0, sys.argv[1])
import paper_1806_03461_amd as T, workloads
sk, ck = T.tfhe_keygen(T.default_params(), workloads.KEY_SEED)
rng = np.random.default_rng(95)
d, p = 11, 5
W = rng.choice(np.array([-1, 0, 1], np.int8), (p, d), p=[0.45, 0.1, 0.45])
Tt = np.array([3, 6, 5, 4, 2], np.int32)
x = rng.integers(0, 2, d).astype(np.uint8)
ctx = T.to_device(T.tfhe_encrypt(sk, 96, x))
h = hashlib.sha256()
for flags in (T.LOWER_MUX_COMPARATOR, T.LOWER_DEFAULT):
    res = torch.empty((p, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted_opts(ck, ctx, d, W, Tt, p, res, 0, flags)
    torch.cuda.synchronize()
    h.update(T.to_host(res).tobytes())
K = (2 * rng.integers(0, 2, (3, 2, 3, 3)) - 1).astype(np.int8)
img = rng.integers(0, 2, 2 * 5 * 4).astype(np.uint8)
res = torch.empty((3 * 5 * 4, 501), dtype=torch.int32, device="cuda")
T.bnn_conv_encrypted(ck, T.to_device(T.tfhe_encrypt(sk, 94, img)), 2, 5, 4, K, np.array([8, 9, 10], np.int32), 1, 1, res)
torch.cuda.synchronize()
h.update(T.to_host(res).tobytes())
s = rng.integers(0, 2, 13).astype(np.uint8)
cs, ca, cb = (T.to_device(T.tfhe_encrypt(sk, 97 + k, s ^ k)) for k in range(3))
out = torch.empty((13, 501), dtype=torch.int32, device="cuda")
T.tfhe_mux_batch(ck, cs, ca, cb, out, 13)
torch.cuda.synchronize()
h.update(T.to_host(out).tobytes())
T.tfhe_gate_batch(ck, "XNOR", ca, cb, out, 13)
torch.cuda.synchronize()
h.update(T.to_host(out).tobytes())
print("digest", h.hexdigest())
"""


def test_launch_chunking_does_not_change_results(gpu):
    """The same calls in a process that splits every launch into chunks of 6 items (levels wider than
    a chunk, multiplexer pairs at chunk boundaries, many launches per batch) give the same bytes
    as with the default chunk size."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    digests = []
    for chunk in (None, "6"):
        env = dict(os.environ)
        env.pop("TFHE_CHUNK_GATES", None)
        if chunk:
            env["TFHE_CHUNK_GATES"] = chunk
        r = subprocess.run([sys.executable, "-c", _CHUNK_SCRIPT, root], env=env, stdout=subprocess.PIPE,
                           stderr=subprocess.STDOUT, text=True, timeout=300)
        assert r.returncode == 0, r.stdout
        digests.append([l for l in r.stdout.splitlines() if l.startswith("digest")][-1])
    assert digests[0] == digests[1]


def test_measured_fp64_ceiling_is_plausible(gpu):
    """The register-resident FMA loop that bench.py quotes the blind rotation against reaches a rate
    between half of and the whole published vector FP64 peak of the device."""
    T, _, ck = gpu
    tflops = T.tfhe_measure_fp64_peak(ck)
    assert 35.0 < tflops < 82.0, tflops


def test_kernel_choices_do_not_change_results(gpu):
    """The same calls give the same bytes whichever kernels serve them: the default process (launches
    this small: latency variant of the blind rotation, matrix-core key switch with split mask words);
    every launch sent to the throughput kernel, with one workgroup per gate and with at most 5
    workgroups (each then walks several gates, the last ones fewer than the first); the gather key
    switch at the benchmark parameters, with a gate's mask words split over workgroups and not; layer
    calls that evaluate their units in groups of at most 300 estimated gates (two or three units)."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    digests = []
    for knobs in ({}, {"TFHE_LATENCY_BATCH": "0", "TFHE_RESIDENT_GROUPS": "5"}, {"TFHE_LATENCY_BATCH": "0"},
                  {"TFHE_KS_MATRIX_FROM": "0"}, {"TFHE_KS_MATRIX_FROM": "0", "TFHE_KS_SPLITS": "1"},
                  {"TFHE_LAYER_GROUP_GATES": "300"}):
        env = dict(os.environ)
        for k in ("TFHE_LATENCY_BATCH", "TFHE_RESIDENT_GROUPS", "TFHE_CHUNK_GATES", "TFHE_KS_MATRIX_FROM", "TFHE_KS_SPLITS",
                  "TFHE_LAYER_GROUP_GATES"):
            env.pop(k, None)
        env.update(knobs)
        r = subprocess.run([sys.executable, "-c", _CHUNK_SCRIPT, root], env=env, stdout=subprocess.PIPE,
                           stderr=subprocess.STDOUT, text=True, timeout=300)
        assert r.returncode == 0, r.stdout
        digests.append([l for l in r.stdout.splitlines() if l.startswith("digest")][-1])
    assert len(set(digests)) == 1, digests


@pytest.mark.parametrize("pattern", ["all_min", "alternating", "random"])
def test_extreme_key_limbs_stay_exact(gpu, orc, pattern):
    """Exactness of the split-integer FP64 products does not depend on the key being 'typical':
    bootstrapping keys whose 16-bit limbs all sit at the ends of their range (imported as raw
    material, they need not encrypt anything) and arbitrary input words give the oracle's bytes,
    and the distance of the raw transform outputs from an integer stays far below 1/2."""
    import torch
    T, _, _ = gpu
    keys = orc.Keys(orc.default_params(), 2024)          # only its arrays and its exact integer arithmetic are used
    rng = np.random.default_rng(77)
    if pattern == "all_min":
        keys.bk[:] = 0x80008000                           # lo limb -32768, hi limb -32767
    elif pattern == "alternating":
        keys.bk[0::2] = 0x7FFF7FFF                        # lo limb +32767, hi limb +32767
        keys.bk[1::2] = 0x80008000
    else:
        keys.bk[:] = rng.integers(0, 1 << 32, keys.bk.size, dtype=np.uint64).astype(np.uint32)
    _, served = T.tfhe_import_keys(T.default_params(), bk_raw=keys.bk, ksk_raw=keys.ksk)
    cnt = 12
    cta = rng.integers(0, 1 << 32, (cnt, 501), dtype=np.uint64).astype(np.uint32)
    ctb = rng.integers(0, 1 << 32, (cnt, 501), dtype=np.uint64).astype(np.uint32)
    T.tfhe_rounding_margin_enable(served, True)
    try:
        got = run_batch(T, served, "XOR", cta, ctb)
        worst = T.tfhe_rounding_margin_read(served)
    finally:
        T.tfhe_rounding_margin_enable(served, False)
    assert np.array_equal(got, oracle_batch(keys, "XOR", cta, ctb))
    assert 0 < worst < 1e-3, worst          # measured: 2.3e-5 at the extreme patterns, 1e-6 for random keys
