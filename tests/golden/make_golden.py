"""Writes tests/golden/sampled_outputs.json: output ciphertexts of sampled units of the
benchmark configurations, computed from scratch by the CPU oracle alone.

Inputs are the seeded synthetic workloads and the oracle's own keys / encryptions; nothing here
touches the GPU library.  Each entry stores the SHA-256 of the expected output ciphertext
(n+1 little-endian uint32 words) and its decryption.  Takes about 15 minutes on 8 cores:

    python tests/golden/make_golden.py [threads]

With "paper" as second argument it writes tests/golden/paper_shapes_outputs.json instead: sampled
outputs of the networks in the shapes of the paper's own models (about 6 minutes on 8 cores):

    python tests/golden/make_golden.py 8 paper
"""
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads                      # noqa: E402
from oracle import circuits as cc     # noqa: E402
from oracle import oracle as orc      # noqa: E402

CFG3_NEURONS = [0, 257]
CFG4_PIXELS = [(0, 0, 0), (5, 0, 13), (17, 13, 27), (31, 27, 27), (9, 14, 14), (20, 27, 3)]
CFG5_L1_NEURONS = [0, 100]


def digest(ct):
    return hashlib.sha256(np.ascontiguousarray(ct, dtype="<u4").tobytes()).hexdigest()


DIABETES_L1_NEURONS = [3]
FACES_L1_PIXELS = [(0, 0, 0), (0, 40, 40), (0, 17, 23)]


def paper_shapes(threads):
    keys = orc.Keys(orc.default_params(), workloads.KEY_SEED)
    out = {"key_seed": workloads.KEY_SEED, "params": list(orc.default_params().as_tuple()), "entries": []}
    t0 = time.time()

    def record(cfg, unit, ct, plain, gates):
        bit = int(keys.decrypt(ct)[0])
        assert bit == int(plain), (cfg, unit, bit, plain)
        out["entries"].append({"cfg": cfg, "unit": unit, "sha256": digest(ct), "bit": bit, "gates": gates})
        print(cfg, unit, "bit", bit, "gates", gates, f"{time.time() - t0:.0f}s", flush=True)

    # cancer shape: the whole network, one entry per score bit (least significant first)
    c = workloads.paper_cancer()
    L = c["layers"][0]
    ct = keys.encrypt(c["x"], c["enc_seed"])
    cir, outs = cc.dense_layer(90, L["W"], None, c["out_bits"])
    res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
    score = int(cc.dense_plain(c["x"], L["W"], None)[0])
    for b in range(c["out_bits"]):
        record("cancer", [b], res[b], (score >> b) & 1, len(cir.gates))

    # diabetes shape: whole first-layer neurons
    c = workloads.paper_diabetes()
    L = c["layers"][0]
    ct = keys.encrypt(c["x"], c["enc_seed"])
    plain = cc.dense_plain(c["x"], L["W"], L["T"])
    for j in DIABETES_L1_NEURONS:
        cir, outs = cc.dense_layer(1704, L["W"][j:j + 1], L["T"][j:j + 1])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("diabetes", [0, j], res[0], plain[j], len(cir.gates))

    # faces shape at one channel: pixels of the first 10x10 convolution
    c = workloads.paper_faces(channels=1)
    L = c["convs"][0]
    ct = keys.encrypt(c["x"].reshape(-1), c["enc_seed"])
    plain = cc.conv_plain(c["x"], L["K"], L["T"], 1, 0)
    for (o, y, x) in FACES_L1_PIXELS:
        cir, outs = cc.conv_layer(1, 50, 50, L["K"], L["T"], 1, 0, pixels=[(o, y, x)])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("faces1", [0, o, y, x], res[0], plain[o, y, x], len(cir.gates))

    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_shapes_outputs.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


def main():
    threads = int(sys.argv[1]) if len(sys.argv) > 1 else (os.cpu_count() or 1)
    if len(sys.argv) > 2 and sys.argv[2] == "paper":
        return paper_shapes(threads)
    keys = orc.Keys(orc.default_params(), workloads.KEY_SEED)
    out = {"key_seed": workloads.KEY_SEED, "params": list(orc.default_params().as_tuple()), "entries": []}

    def record(cfg, unit, ct, plain, gates):
        bit = int(keys.decrypt(ct)[0])
        assert bit == int(plain), (cfg, unit, bit, plain)
        out["entries"].append({"cfg": cfg, "unit": unit, "sha256": digest(ct), "bit": bit, "gates": gates})
        print(cfg, unit, "bit", bit, "gates", gates, f"{time.time() - t0:.0f}s", flush=True)

    t0 = time.time()
    # cfg 2: one neuron, its seeded threshold and the fixed threshold 128 on the same popcount
    c = workloads.cfg2()
    ct = keys.encrypt(c["x"], c["enc_seed"])
    for T in (int(c["T"][0]), 128):
        cir, outs = cc.dense_layer(256, c["W"], np.array([T], np.int32))
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("cfg2", [T], res[0], cc.dense_plain(c["x"], c["W"], np.array([T]))[0], len(cir.gates))

    # cfg 3: whole neurons of the 784 -> 512 layer
    c = workloads.cfg3()
    ct = keys.encrypt(c["x"], c["enc_seed"])
    plain = cc.dense_plain(c["x"], c["W"], c["T"])
    for j in CFG3_NEURONS:
        cir, outs = cc.dense_layer(784, c["W"][j:j + 1], c["T"][j:j + 1])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("cfg3", [j], res[0], plain[j], len(cir.gates))

    # cfg 4: output pixels of the 3x3 convolution, corners and edges included
    c = workloads.cfg4()
    ct = keys.encrypt(c["x"].reshape(-1), c["enc_seed"])
    plain = cc.conv_plain(c["x"], c["K"], c["T"], 1, 1)
    for (o, y, x) in CFG4_PIXELS:
        cir, outs = cc.conv_layer(16, 28, 28, c["K"], c["T"], 1, 1, pixels=[(o, y, x)])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("cfg4", [o, y, x], res[0], plain[o, y, x], len(cir.gates))

    # cfg 5: first-layer neurons of the sparsified MLP (later layers need the whole first layer)
    c = workloads.cfg5()
    ct = keys.encrypt(c["x"], c["enc_seed"])
    L1 = c["layers"][0]
    plain = cc.dense_plain(c["x"], L1["W"], L1["T"])
    for j in CFG5_L1_NEURONS:
        cir, outs = cc.dense_layer(784, L1["W"][j:j + 1], L1["T"][j:j + 1])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("cfg5", [0, j], res[0], plain[j], len(cir.gates))

    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "sampled_outputs.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
