"""GPU parity on whole networks in the shapes of the paper's own models (Sec. 5.2: Cancer
FC 90->1; Diabetes FC 1704->10, sign, FC 10->3; Faces five 10x10 convolutions on 50x50 and
FC 25->1), with synthetic weights.  The Faces shape runs at one channel here, the structure and
the image size being the paper's.

Evidence per network: sampled first-layer units against digests the CPU oracle computed from
scratch (tests/golden/paper_shapes_outputs.json); every activation of every layer decrypted
against the exact integer network; whole units of the later layers re-evaluated by the oracle on
the GPU's own activations, bit for bit.
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
GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_shapes_outputs.json")


def digest(ct):
    return hashlib.sha256(np.ascontiguousarray(ct, dtype="<u4").tobytes()).hexdigest()


@pytest.fixture(scope="module")
def golden():
    g = json.load(open(GOLD))
    assert g["key_seed"] == workloads.KEY_SEED
    return {(e["cfg"], tuple(e["unit"])): e for e in g["entries"]}


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_1806_03461_amd as T
    sk, ck = T.tfhe_keygen(T.default_params(), workloads.KEY_SEED)
    T.tfhe_cloud_key_upload(ck)
    return T, sk, ck


def scores(bits, out_bits):
    return (bits.reshape(-1, out_bits).astype(np.int64) << np.arange(out_bits)).sum(axis=1)


def test_cancer_shape_whole_network_bit_exact(gpu, golden):
    import torch
    T, sk, ck = gpu
    c = workloads.paper_cancer()
    L, ob = c["layers"][0], c["out_bits"]
    x = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"]))
    out = torch.empty((ob, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted(ck, x, 90, L["W"], None, 1, out, ob)
    torch.cuda.synchronize()
    got = T.to_host(out)
    for b in range(ob):
        assert digest(got[b]) == golden[("cancer", (b,))]["sha256"], b
    assert scores(T.tfhe_decrypt(sk, got), ob)[0] == cc.dense_plain(c["x"], L["W"], None)[0]


def test_diabetes_shape_two_layers(gpu, golden, real_keys):
    import torch
    T, sk, ck = gpu
    c = workloads.paper_diabetes()
    L1, L2, ob = c["layers"][0], c["layers"][1], c["out_bits"]
    x = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"]))
    h = torch.empty((10, 501), dtype=torch.int32, device="cuda")
    out = torch.empty((3 * ob, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted(ck, x, 1704, L1["W"], L1["T"], 10, h)
    T.bnn_dense_encrypted(ck, h, 10, L2["W"], None, 3, out, ob)
    torch.cuda.synchronize()
    hh, got = T.to_host(h), T.to_host(out)
    # first layer: a whole neuron from scratch, every neuron against the integer layer
    assert digest(hh[3]) == golden[("diabetes", (0, 3))]["sha256"]
    p1 = cc.dense_plain(c["x"], L1["W"], L1["T"])
    assert np.array_equal(T.tfhe_decrypt(sk, hh), p1)
    # second layer: the oracle's whole layer on the GPU's hidden ciphertexts
    cir, outs = cc.dense_layer(10, L2["W"], None, ob)
    ref, _ = cc.eval_encrypted(real_keys, cir, hh, outs, threads=16)
    assert np.array_equal(got, ref)
    assert np.array_equal(scores(T.tfhe_decrypt(sk, got), ob), cc.dense_plain(p1, L2["W"], None))


def test_faces_shape_one_channel(gpu, golden, real_keys, say):
    import torch
    T, sk, ck = gpu
    c = workloads.paper_faces(channels=1)
    ob = c["out_bits"]
    acts = [T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"].reshape(-1)))]
    plain, shapes = [c["x"]], [c["x"].shape]
    for li, L in enumerate(c["convs"]):
        C_, H, Wd = shapes[-1]
        plain.append(cc.conv_plain(plain[-1], L["K"], L["T"], 1, 0))
        shapes.append(plain[-1].shape)
        out = torch.empty((plain[-1].size, 501), dtype=torch.int32, device="cuda")
        say(f"[faces] convolution {li + 1}: {shapes[-2]} -> {shapes[-1]}")
        T.bnn_conv_encrypted(ck, acts[-1], C_, H, Wd, L["K"], L["T"], 1, 0, out)
        torch.cuda.synchronize()
        acts.append(out)
    assert [s[1] for s in shapes] == [50, 41, 32, 23, 14, 5]
    D = c["dense"]
    out = torch.empty((ob, 501), dtype=torch.int32, device="cuda")
    T.bnn_dense_encrypted(ck, acts[-1], 25, D["W"], None, 1, out, ob)
    torch.cuda.synchronize()
    host = [T.to_host(a) for a in acts]
    final = T.to_host(out)
    # every activation of every layer against the integer network
    for li in range(1, 6):
        assert np.array_equal(T.tfhe_decrypt(sk, host[li]).reshape(shapes[li]), plain[li]), li
    assert scores(T.tfhe_decrypt(sk, final), ob)[0] == cc.dense_plain(plain[5].reshape(-1), D["W"], None)[0]
    # first convolution: pixels from scratch
    for (o, y, xx) in ((0, 0, 0), (0, 40, 40), (0, 17, 23)):
        assert digest(host[1][(o * 41 + y) * 41 + xx]) == golden[("faces1", (0, o, y, xx))]["sha256"], (y, xx)
    # later convolutions: one pixel each, the oracle fed with the GPU's activations
    for li, (y, xx) in ((1, (31, 0)), (2, (11, 22)), (3, (0, 13)), (4, (4, 4))):
        L = c["convs"][li]
        C_, H, Wd = shapes[li]
        say(f"[faces] oracle pixel of convolution {li + 1}")
        cir, outs = cc.conv_layer(C_, H, Wd, L["K"], L["T"], 1, 0, pixels=[(0, y, xx)])
        ref, _ = cc.eval_encrypted(real_keys, cir, host[li], outs, threads=16)
        assert np.array_equal(host[li + 1][y * shapes[li + 1][2] + xx], ref[0]), (li, y, xx)
    # the last layer whole
    cir, outs = cc.dense_layer(25, D["W"], None, ob)
    ref, _ = cc.eval_encrypted(real_keys, cir, host[5], outs, threads=16)
    assert np.array_equal(final, ref)


def test_faces_shape_first_convolution_at_32_channels(gpu, golden, say):
    """The first convolution of the Faces shape at the paper's width (Sec. 5.2: 32 output channels,
    10 x 10 windows on the 50 x 50 image): 53,792 units, 36 M gates, evaluated eight output channels
    per call so that a step of the work ends, and says so, every 40 s (bench.py times the layer as
    one call).  Every output pixel is decrypted against the integer layer; six pixels are compared
    with digests the oracle computed from scratch.  (The later convolutions at this width read 3,200
    inputs per unit, 732 M gates each, about fifty minutes of GPU time per layer: they run at
    reduced width in the test above.)"""
    import torch
    T, sk, ck = gpu
    c = workloads.paper_faces(channels=32)
    L = c["convs"][0]
    x = T.to_device(T.tfhe_encrypt(sk, c["enc_seed"], c["x"].reshape(-1)))
    plain = cc.conv_plain(c["x"], L["K"], L["T"], 1, 0)
    assert plain.shape == (32, 41, 41)
    out = torch.empty((plain.size, 501), dtype=torch.int32, device="cuda")
    say("[faces32] first convolution: (1, 50, 50) -> (32, 41, 41)")
    gates = 0
    for o0 in range(0, 32, 8):
        K = np.ascontiguousarray(L["K"][o0:o0 + 8])
        Th = np.ascontiguousarray(L["T"][o0:o0 + 8])
        T.bnn_conv_encrypted(ck, x, 1, 50, 50, K, Th, 1, 0, out[o0 * 41 * 41:(o0 + 8) * 41 * 41])
        torch.cuda.synchronize()
        st = T.tfhe_last_layer_stats(ck)
        gates += st["gates"]
        say(f"[faces32] output channels {o0}..{o0 + 7}: {st['gates']} gates, {st['depths']} depths, "
            f"wire pool {st['pool_wires']} of {st['circuit_wires']} wires")
    assert gates > 30_000_000
    got = T.to_host(out)
    assert np.array_equal(T.tfhe_decrypt(sk, got).reshape(plain.shape), plain)
    for (o, y, xx) in ((0, 0, 0), (13, 40, 40), (31, 17, 23), (7, 0, 40), (22, 40, 0), (18, 20, 20)):
        assert digest(got[(o * 41 + y) * 41 + xx]) == golden[("faces32", (0, o, y, xx))]["sha256"], (o, y, xx)
