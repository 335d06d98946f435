"""GPU parity on the five benchmark configurations at full size, in the launch configuration
the benchmark times.

Three kinds of evidence, strongest first:
  1. sampled whole units (neurons / pixels) against tests/golden/sampled_outputs.json, which the
     CPU oracle computed from scratch from the seeded inputs (bit-exact ciphertext digests);
  2. every output of every configuration decrypted and compared with the exact integer layer;
  3. a local property that holds at any size: randomly sampled gates deep inside the circuit,
     re-evaluated by the oracle on the GPU's own input wires, give the GPU's output wire bytes.
"""
import hashlib
import json
import os
import sys

import numpy as np
import pytest

import workloads
from oracle import circuits as cc

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden", "sampled_outputs.json")


def digest(ct):
    return hashlib.sha256(np.ascontiguousarray(ct, dtype="<u4").tobytes()).hexdigest()


@pytest.fixture(scope="module")
def golden():
    g = json.load(open(GOLD))
    assert g["key_seed"] == workloads.KEY_SEED
    table = {}
    for e in g["entries"]:
        table[(e["cfg"], tuple(e["unit"]))] = e
    return table


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1806_03461_amd as T
    sk, ck = T.tfhe_keygen(T.default_params(), workloads.KEY_SEED)
    T.tfhe_cloud_key_upload(ck)
    return T, sk, ck


def test_cfg2_one_neuron_bit_exact(gpu, golden):
    import torch
    T, sk, ck = gpu
    c = workloads.cfg2()
    x = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"]))
    out = torch.empty((1, 501), dtype=torch.int32, device="cuda")
    for Tt in (int(c["T"][0]), 128):
        T.bnn_dense_encrypted(ck, x, 256, c["W"], np.array([Tt], np.int32), 1, out)
        torch.cuda.synchronize()
        got = T.to_host(out)[0]
        e = golden[("cfg2", (Tt,))]
        assert digest(got) == e["sha256"]
        assert T.tfhe_decrypt(sk, got)[0] == e["bit"] == cc.dense_plain(c["x"], c["W"], np.array([Tt]))[0]


def test_cfg3_dense_layer(gpu, golden, real_keys):
    import torch
    T, sk, ck = gpu
    c = workloads.cfg3()
    ctx = T.tfhe_encrypt(sk, c["enc_seed"], c["x"])
    gates, outs, nw = T.bnn_dense_lower(784, c["W"], c["T"], 512)
    wires = torch.zeros((nw, 501), dtype=torch.int32, device="cuda")
    wires[:784] = T.to_device(ctx)
    wires[784] = T.to_device(T.tfhe_trivial(T.default_params(), 0).reshape(1, -1))[0]
    wires[785] = T.to_device(T.tfhe_trivial(T.default_params(), 1).reshape(1, -1))[0]
    T.tfhe_gate_stream(ck, gates, wires, nw)
    torch.cuda.synchronize()
    assert (outs["wire"] >= 0).all()
    idx = torch.from_numpy(outs["wire"].astype(np.int64)).cuda()
    out = T.to_host(wires[idx])
    neg = outs["value"].astype(bool)
    out[neg] = (0 - out[neg]).astype(np.uint32)
    # (2) all 512 outputs against the integer layer
    assert np.array_equal(T.tfhe_decrypt(sk, out), cc.dense_plain(c["x"], c["W"], c["T"]))
    # (1) whole neurons computed from scratch by the oracle
    for j in (0, 257, 100, 511):
        assert digest(out[j]) == golden[("cfg3", (j,))]["sha256"], j
    # the layer entry point (wire pool with recycled slots) gives the same 512 ciphertexts
    res = torch.empty((512, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted(ck, T.to_device(ctx), 784, c["W"], c["T"], 512, res)
    torch.cuda.synchronize()
    assert np.array_equal(T.to_host(res), out)
    st = T.tfhe_last_layer_stats(ck)
    assert st["gates"] == len(gates) and st["depths"] == 36 and st["pool_wires"] < 0.45 * nw
    # (3) 256 random gates anywhere in the circuit, oracle on the GPU's input wires
    rng = np.random.default_rng(33)
    pick = np.sort(rng.choice(len(gates), 256, replace=False))
    sel = gates[pick]
    take = lambda w: T.to_host(wires[torch.from_numpy(w.astype(np.int64)).cuda()])
    k = len(sel)
    work = np.concatenate([take(sel["in0"]), take(sel["in1"]), np.zeros((k, 501), np.uint32)])
    recs = sel.copy()
    recs["in0"], recs["in1"], recs["out"] = np.arange(k), k + np.arange(k), 2 * k + np.arange(k)
    real_keys.gate_batch(recs, work, threads=16)
    assert np.array_equal(work[2 * k:], take(sel["out"]))


CFG4_PIXELS = [(0, 0, 0), (5, 0, 13), (17, 13, 27), (31, 27, 27), (9, 14, 14), (20, 27, 3),
               (1, 0, 27), (2, 27, 0), (3, 13, 0), (4, 27, 14), (6, 0, 1), (7, 1, 0), (8, 26, 27), (10, 27, 26),
               (11, 1, 1), (12, 26, 26), (13, 7, 19), (14, 19, 7), (15, 12, 15), (16, 3, 24), (18, 24, 3),
               (19, 10, 10), (21, 17, 22), (22, 22, 17), (23, 5, 5), (24, 15, 12), (25, 8, 21), (26, 21, 8),
               (27, 13, 13), (28, 2, 16), (29, 16, 2), (30, 25, 11)]


def test_cfg4_conv_layer(gpu, golden, real_keys, capsys):
    import torch
    T, sk, ck = gpu

    def say(msg):
        with capsys.disabled():
            sys.stderr.write(f"[cfg4] {msg}\n")
            sys.stderr.flush()

    c = workloads.cfg4()
    x = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"].reshape(-1)))
    out = torch.empty((32 * 28 * 28, 501), dtype=torch.int32, device="cuda")
    # the whole layer as one call: 25,088 units, 24.4 M gates
    T.bnn_conv_encrypted(ck, x, 16, 28, 28, c["K"], c["T"], 1, 1, out)
    torch.cuda.synchronize()
    st = T.tfhe_last_layer_stats(ck)
    say(f"one call done: {st['gates']} gates, {st['depths']} depths, wire pool {st['pool_wires']} of "
        f"{st['circuit_wires']} wires ({st['pool_wires'] * 2004 / 1e9:.1f} GB)")
    assert st["gates"] > 24_000_000 and st["pool_wires"] < 0.45 * st["circuit_wires"]
    got = T.to_host(out)
    # (2) every output pixel against the integer layer
    plain = cc.conv_plain(c["x"], c["K"], c["T"], 1, 1)
    assert np.array_equal(T.tfhe_decrypt(sk, got).reshape(32, 28, 28), plain)
    # (1) 32 pixels computed from scratch by the oracle: corners, edges, interior, every channel
    for (o, y, xx) in CFG4_PIXELS:
        assert digest(got[(o * 28 + y) * 28 + xx]) == golden[("cfg4", (o, y, xx))]["sha256"], (o, y, xx)
    # (3) eight output channels again as a gate stream on wires the test owns (no slot reuse): the
    # same output bytes, and 256 random gates anywhere in it re-evaluated by the oracle on the GPU's wires
    ch = slice(8, 16)
    gates, outs, nw = T.bnn_conv_lower(16, 28, 28, c["K"][ch], c["T"][ch], 1, 1)
    wires = torch.zeros((nw, 501), dtype=torch.int32, device="cuda")
    nin = 16 * 28 * 28
    wires[:nin] = x
    wires[nin] = T.to_device(T.tfhe_trivial(T.default_params(), 0).reshape(1, -1))[0]
    wires[nin + 1] = T.to_device(T.tfhe_trivial(T.default_params(), 1).reshape(1, -1))[0]
    T.tfhe_gate_stream(ck, gates, wires, nw)
    torch.cuda.synchronize()
    say(f"gate stream of channels 8..15 done ({len(gates)} gates)")
    take = lambda w: T.to_host(wires[torch.from_numpy(w.astype(np.int64)).cuda()])
    assert (outs["wire"] >= nin + 2).all()
    slice_out = take(outs["wire"])
    neg = outs["value"].astype(bool)
    slice_out[neg] = (0 - slice_out[neg]).astype(np.uint32)
    assert np.array_equal(slice_out, got[8 * 784:16 * 784])
    rng = np.random.default_rng(44)
    pick = np.sort(rng.choice(len(gates), 256, replace=False))
    sel = gates[pick]
    k = len(sel)
    work = np.concatenate([take(sel["in0"]), take(sel["in1"]), np.zeros((k, 501), np.uint32)])
    recs = sel.copy()
    recs["in0"], recs["in1"], recs["out"] = np.arange(k), k + np.arange(k), 2 * k + np.arange(k)
    real_keys.gate_batch(recs, work, threads=16)
    assert np.array_equal(work[2 * k:], take(sel["out"]))


def test_cfg5_sparse_mlp(gpu, golden, real_keys):
    import torch
    T, sk, ck = gpu
    c = workloads.cfg5()
    h = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"]))
    acts = [h]
    plain = [c["x"]]
    for li, layer in enumerate(c["layers"]):
        p, d = layer["W"].shape
        last = layer["T"] is None
        out = torch.empty((p * (c["out_bits"] if last else 1), 501), dtype=torch.int32, device="cuda")
        T.bnn_dense_encrypted(ck, acts[-1], d, layer["W"], layer["T"], p, out, c["out_bits"] if last else 0)
        acts.append(out)
        plain.append(cc.dense_plain(plain[-1], layer["W"], layer["T"]))
    torch.cuda.synchronize()
    host = [T.to_host(a) for a in acts]
    # (2) every activation of every layer against the plain integer network
    for li in (1, 2):
        assert np.array_equal(T.tfhe_decrypt(sk, host[li]), plain[li]), li
    bits = T.tfhe_decrypt(sk, host[3]).reshape(10, c["out_bits"]).astype(np.int64)
    assert np.array_equal((bits << np.arange(c["out_bits"])).sum(axis=1), plain[3])
    # (1) first-layer neurons from scratch
    for j in (0, 100):
        assert digest(host[1][j]) == golden[("cfg5", (0, j))]["sha256"], j
    # (3) two whole units of each later layer, oracle fed with the GPU's activations
    for li, j in ((1, 7), (1, 200), (2, 3), (2, 9)):
        layer = c["layers"][li]
        last = layer["T"] is None
        cir, outs = cc.dense_layer(layer["W"].shape[1], layer["W"][j:j + 1],
                                   None if last else layer["T"][j:j + 1], c["out_bits"])
        ref, _ = cc.eval_encrypted(real_keys, cir, host[li], outs, threads=16)
        mine = host[li + 1][j * c["out_bits"]:(j + 1) * c["out_bits"]] if last else host[li + 1][j:j + 1]
        assert np.array_equal(mine, ref), (li, j)


def test_degenerate_units(gpu, real_keys):
    """Constant outputs (T <= 0, T > m, all-zero row), a single (negated) input passed through
    without any gate, and a layer with no gates at all."""
    import torch
    T, sk, ck = gpu
    x = np.array([1, 0, 1, 1, 0], np.uint8)
    ctx = T.tfhe_encrypt(sk, 61, x)
    W = np.array([[0, 0, 0, 0, 0], [0, -1, 0, 0, 0], [1, 1, 1, 1, 1], [1, -1, 1, 1, -1], [0, 0, 1, 0, 0]], np.int8)
    Tt = np.array([0, 1, 6, -3, 1], np.int32)
    for rows in ([0, 1, 4], [0, 1, 2, 3, 4]):
        p = len(rows)
        out = torch.empty((p, 501), dtype=torch.int32, device="cuda")
        T.bnn_dense_encrypted(ck, T.to_device(ctx), 5, W[rows], Tt[rows], p, out)
        torch.cuda.synchronize()
        got = T.to_host(out)
        cir, o = cc.dense_layer(5, W[rows], Tt[rows])
        ref, _ = cc.eval_encrypted(real_keys, cir, ctx, o, threads=4)
        if p == 3:
            assert len(cir.gates) == 0 and len(T.bnn_dense_lower(5, W[rows], Tt[rows], p)[0]) == 0
        assert np.array_equal(got, ref)
        assert np.array_equal(got[1], (0 - ctx[1]).astype(np.uint32)) and np.array_equal(got[-1], ctx[2])
        assert list(T.tfhe_decrypt(sk, got)) == list(cc.dense_plain(x, W[rows], Tt[rows]))
    assert list(cc.dense_plain(x, W, Tt)) == [1, 1, 0, 1, 1]


def test_small_convolution_entry_point(gpu, real_keys):
    """Stride 2 and stride 1 on a 2x6x5 image: every pixel's ciphertext against the oracle's own
    lowering (3 + 12 pixels of 18 taps each)."""
    import torch
    T, sk, ck = gpu
    rng = np.random.default_rng(71)
    x = rng.integers(0, 2, (2, 6, 5)).astype(np.uint8)
    K = (2 * rng.integers(0, 2, (2, 2, 3, 3)) - 1).astype(np.int8)
    K[0, 1, 1, 1] = 0
    Tt = np.array([8, 10], np.int32)
    ctx = T.tfhe_encrypt(sk, 72, x.reshape(-1))
    for stride, pad, pixels in ((2, 0, None), (1, 1, [(0, 0, 0), (1, 5, 4), (0, 2, 2), (1, 0, 3)])):
        Ho, Wo = (6 + 2 * pad - 3) // stride + 1, (5 + 2 * pad - 3) // stride + 1
        out = torch.empty((2 * Ho * Wo, 501), dtype=torch.int32, device="cuda")
        T.bnn_conv_encrypted(ck, T.to_device(ctx), 2, 6, 5, K, Tt, stride, pad, out)
        torch.cuda.synchronize()
        got = T.to_host(out)
        assert np.array_equal(T.tfhe_decrypt(sk, got).reshape(2, Ho, Wo), cc.conv_plain(x, K, Tt, stride, pad))
        cir, o = cc.conv_layer(2, 6, 5, K, Tt, stride, pad, pixels=pixels)
        ref, _ = cc.eval_encrypted(real_keys, cir, ctx, o, threads=16)
        if pixels is None:
            assert np.array_equal(got, ref)
        else:
            for k, (oc, y, xx) in enumerate(pixels):
                assert np.array_equal(got[(oc * Ho + y) * Wo + xx], ref[k])


def test_plus_one_trick_layers(gpu, real_keys):
    """The '+1' lowering: small dense and convolution layers byte for byte against the oracle's own
    '+1' circuits; the full 784 -> 512 layer decrypted against the integer layer."""
    import torch
    T, sk, ck = gpu
    rng = np.random.default_rng(101)
    d, p = 13, 4
    W = (2 * rng.integers(0, 2, (p, d)) - 1).astype(np.int8)
    W[3, 2] = 0                                            # falls back to the plain unit
    Tt = np.array([5, 7, 9, 6], np.int32)
    x = rng.integers(0, 2, d).astype(np.uint8)
    ctx = T.tfhe_encrypt(sk, 102, x)
    out = torch.empty((p, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted_opts(ck, T.to_device(ctx), d, W, Tt, p, out, 0, T.LOWER_PLUS_ONE)
    torch.cuda.synchronize()
    cir, o = cc.dense_layer(d, W, Tt, plus_one=True)
    ref, _ = cc.eval_encrypted(real_keys, cir, ctx, o, threads=16)
    assert np.array_equal(T.to_host(out), ref)
    assert np.array_equal(T.tfhe_decrypt(sk, T.to_host(out)), cc.dense_plain(x, W, Tt))

    xi = rng.integers(0, 2, (2, 4, 3)).astype(np.uint8)
    K = (2 * rng.integers(0, 2, (3, 2, 3, 3)) - 1).astype(np.int8)
    Tc = np.array([8, 9, 10], np.int32)
    cti = T.tfhe_encrypt(sk, 103, xi.reshape(-1))
    outc = torch.empty((3 * 4 * 3, 501), dtype=torch.int32, device="cuda")
    T.bnn_conv_encrypted_opts(ck, T.to_device(cti), 2, 4, 3, K, Tc, 1, 1, outc, T.LOWER_PLUS_ONE)
    torch.cuda.synchronize()
    pixels = [(0, 0, 0), (2, 3, 2), (1, 1, 1)]
    cir, o = cc.conv_layer(2, 4, 3, K, Tc, 1, 1, pixels=pixels, plus_one=True)
    ref, _ = cc.eval_encrypted(real_keys, cir, cti, o, threads=16)
    got = T.to_host(outc)
    for k, (oc, y, xx) in enumerate(pixels):
        assert np.array_equal(got[(oc * 4 + y) * 3 + xx], ref[k])
    assert np.array_equal(T.tfhe_decrypt(sk, got).reshape(3, 4, 3), cc.conv_plain(xi, K, Tc, 1, 1))

    c = workloads.cfg3()
    xd = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"]))
    big = torch.empty((512, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted_opts(ck, xd, 784, c["W"], c["T"], 512, big, 0, T.LOWER_PLUS_ONE)
    torch.cuda.synchronize()
    assert np.array_equal(T.tfhe_decrypt(sk, T.to_host(big)), cc.dense_plain(c["x"], c["W"], c["T"]))


def test_shared_gate_lowering(gpu, real_keys):
    """Gate sharing across units: a small layer byte for byte against the oracle's shared
    circuit, and the full 784 -> 512 layer ('+1' trick and sharing together: 1.04 M gates instead
    of 2.79 M) decrypted against the integer layer."""
    import torch
    T, sk, ck = gpu
    rng = np.random.default_rng(111)
    d, p = 16, 6
    W = (2 * rng.integers(0, 2, (p, d)) - 1).astype(np.int8)
    Tt = rng.integers(5, 12, p).astype(np.int32)
    x = rng.integers(0, 2, d).astype(np.uint8)
    ctx = T.tfhe_encrypt(sk, 112, x)
    out = torch.empty((p, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted_opts(ck, T.to_device(ctx), d, W, Tt, p, out, 0, T.LOWER_SHARE_GATES)
    torch.cuda.synchronize()
    cir, o = cc.dense_layer(d, W, Tt, share=True)
    assert len(cir.gates) < len(cc.dense_layer(d, W, Tt)[0].gates)
    ref, _ = cc.eval_encrypted(real_keys, cir, ctx, o, threads=16)
    assert np.array_equal(T.to_host(out), ref)
    c = workloads.cfg3()
    xd = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"]))
    big = torch.empty((512, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted_opts(ck, xd, 784, c["W"], c["T"], 512, big, 0, T.LOWER_SHARE_GATES | T.LOWER_PLUS_ONE)
    torch.cuda.synchronize()
    assert np.array_equal(T.tfhe_decrypt(sk, T.to_host(big)), cc.dense_plain(c["x"], c["W"], c["T"]))


def test_sorting_network_layer(gpu, real_keys):
    """The sorting-network inner product on the GPU against the oracle's own network, byte for byte."""
    import torch
    T, sk, ck = gpu
    rng = np.random.default_rng(121)
    d, p = 12, 3
    W = rng.choice(np.array([-1, 0, 1], np.int8), (p, d), p=[0.45, 0.1, 0.45])
    Tt = np.array([3, 6, 5], np.int32)
    x = rng.integers(0, 2, d).astype(np.uint8)
    ctx = T.tfhe_encrypt(sk, 122, x)
    out = torch.empty((p, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted_opts(ck, T.to_device(ctx), d, W, Tt, p, out, 0, T.LOWER_SORTING_NETWORK)
    torch.cuda.synchronize()
    cir, o = cc.dense_layer(d, W, Tt, comparator="sort")
    ref, _ = cc.eval_encrypted(real_keys, cir, ctx, o, threads=16)
    assert np.array_equal(T.to_host(out), ref)
    assert np.array_equal(T.tfhe_decrypt(sk, T.to_host(out)), cc.dense_plain(x, W, Tt))
