"""Writes tests/golden/sampled_outputs.json: output ciphertexts of sampled units of the
benchmark configurations, computed from scratch by the CPU oracle alone.

Inputs are the seeded synthetic workloads and the oracle's own keys / encryptions; nothing here
touches the GPU library.  Each entry stores the SHA-256 of the expected output ciphertext
(n+1 little-endian uint32 words) and its decryption.  Takes about 20 minutes on 8 cores:

    python tests/golden/make_golden.py [threads]

Entries that the output file already holds (written by an earlier run of this script) are kept
and not recomputed; delete the file to recompute everything.

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

CFG3_NEURONS = [0, 257, 100, 511]
# 32 output pixels (channel, row, column) of the 28 x 28 map: the four corners, pixels on each of
# the four edges (their windows reach into the padding), and interior pixels; every channel once
CFG4_PIXELS = [(0, 0, 0), (5, 0, 13), (17, 13, 27), (31, 27, 27), (9, 14, 14), (20, 27, 3),
               (1, 0, 27), (2, 27, 0), (3, 13, 0), (4, 27, 14), (6, 0, 1), (7, 1, 0), (8, 26, 27), (10, 27, 26),
               (11, 1, 1), (12, 26, 26), (13, 7, 19), (14, 19, 7), (15, 12, 15), (16, 3, 24), (18, 24, 3),
               (19, 10, 10), (21, 17, 22), (22, 22, 17), (23, 5, 5), (24, 15, 12), (25, 8, 21), (26, 21, 8),
               (27, 13, 13), (28, 2, 16), (29, 16, 2), (30, 25, 11)]
CFG5_L1_NEURONS = [0, 100]


def digest(ct):
    return hashlib.sha256(np.ascontiguousarray(ct, dtype="<u4").tobytes()).hexdigest()


DIABETES_L1_NEURONS = [3]
FACES_L1_PIXELS = [(0, 0, 0), (0, 40, 40), (0, 17, 23)]
# the first convolution at the paper's 32 channels: (channel, row, column) of the 41 x 41 map
FACES32_L1_PIXELS = [(0, 0, 0), (13, 40, 40), (31, 17, 23), (7, 0, 40), (22, 40, 0), (18, 20, 20)]


def paper_shapes(threads):
    keys = orc.Keys(orc.default_params(), workloads.KEY_SEED)
    out = {"key_seed": workloads.KEY_SEED, "params": list(orc.default_params().as_tuple()), "entries": []}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_shapes_outputs.json")
    have = {}
    if os.path.exists(path):
        old = json.load(open(path))
        if old.get("key_seed") == out["key_seed"] and old.get("params") == out["params"]:
            have = {(e["cfg"], tuple(e["unit"])): e for e in old["entries"]}
    t0 = time.time()

    def known(cfg, unit):
        e = have.get((cfg, tuple(unit)))
        if e is not None:
            out["entries"].append(e)
            print(cfg, unit, "kept", flush=True)
        return e is not None

    def record(cfg, unit, ct, plain, gates):
        bit = int(keys.decrypt(ct)[0])
        assert bit == int(plain), (cfg, unit, bit, plain)
        out["entries"].append({"cfg": cfg, "unit": unit, "sha256": digest(ct), "bit": bit, "gates": gates})
        print(cfg, unit, "bit", bit, "gates", gates, f"{time.time() - t0:.0f}s", flush=True)

    # cancer shape: the whole network, one entry per score bit (least significant first)
    c = workloads.paper_cancer()
    L = c["layers"][0]
    if not all(known("cancer", [b]) for b in range(c["out_bits"])):
        out["entries"] = [e for e in out["entries"] if e["cfg"] != "cancer"]
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
        if known("diabetes", [0, j]):
            continue
        cir, outs = cc.dense_layer(1704, L["W"][j:j + 1], L["T"][j:j + 1])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("diabetes", [0, j], res[0], plain[j], len(cir.gates))

    # faces shape at one channel: pixels of the first 10x10 convolution
    c = workloads.paper_faces(channels=1)
    L = c["convs"][0]
    ct = keys.encrypt(c["x"].reshape(-1), c["enc_seed"])
    plain = cc.conv_plain(c["x"], L["K"], L["T"], 1, 0)
    for (o, y, x) in FACES_L1_PIXELS:
        if known("faces1", [0, o, y, x]):
            continue
        cir, outs = cc.conv_layer(1, 50, 50, L["K"], L["T"], 1, 0, pixels=[(o, y, x)])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("faces1", [0, o, y, x], res[0], plain[o, y, x], len(cir.gates))

    # faces shape at the paper's 32 channels: pixels of the first convolution (1 -> 32 channels)
    c = workloads.paper_faces(channels=32)
    L = c["convs"][0]
    ct = keys.encrypt(c["x"].reshape(-1), c["enc_seed"])
    plain = cc.conv_plain(c["x"], L["K"], L["T"], 1, 0)
    for (o, y, x) in FACES32_L1_PIXELS:
        if known("faces32", [0, o, y, x]):
            continue
        cir, outs = cc.conv_layer(1, 50, 50, L["K"], L["T"], 1, 0, pixels=[(o, y, x)])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("faces32", [0, o, y, x], res[0], plain[o, y, x], len(cir.gates))

    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


def main():
    threads = int(sys.argv[1]) if len(sys.argv) > 1 else (os.cpu_count() or 1)
    if len(sys.argv) > 2 and sys.argv[2] == "paper":
        return paper_shapes(threads)
    keys = orc.Keys(orc.default_params(), workloads.KEY_SEED)
    out = {"key_seed": workloads.KEY_SEED, "params": list(orc.default_params().as_tuple()), "entries": []}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "sampled_outputs.json")
    have = {}
    if os.path.exists(path):
        old = json.load(open(path))
        if old.get("key_seed") == out["key_seed"] and old.get("params") == out["params"]:
            have = {(e["cfg"], tuple(e["unit"])): e for e in old["entries"]}

    def known(cfg, unit):
        e = have.get((cfg, tuple(unit)))
        if e is not None:
            out["entries"].append(e)
            print(cfg, unit, "kept", flush=True)
        return e is not None

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
        if known("cfg2", [T]):
            continue
        cir, outs = cc.dense_layer(256, c["W"], np.array([T], np.int32))
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("cfg2", [T], res[0], cc.dense_plain(c["x"], c["W"], np.array([T]))[0], len(cir.gates))

    # cfg 3: whole neurons of the 784 -> 512 layer
    c = workloads.cfg3()
    ct = keys.encrypt(c["x"], c["enc_seed"])
    plain = cc.dense_plain(c["x"], c["W"], c["T"])
    for j in CFG3_NEURONS:
        if known("cfg3", [j]):
            continue
        cir, outs = cc.dense_layer(784, c["W"][j:j + 1], c["T"][j:j + 1])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("cfg3", [j], res[0], plain[j], len(cir.gates))

    # cfg 4: output pixels of the 3x3 convolution, corners and edges included
    c = workloads.cfg4()
    ct = keys.encrypt(c["x"].reshape(-1), c["enc_seed"])
    plain = cc.conv_plain(c["x"], c["K"], c["T"], 1, 1)
    for (o, y, x) in CFG4_PIXELS:
        if known("cfg4", [o, y, x]):
            continue
        cir, outs = cc.conv_layer(16, 28, 28, c["K"], c["T"], 1, 1, pixels=[(o, y, x)])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("cfg4", [o, y, x], res[0], plain[o, y, x], len(cir.gates))

    # cfg 5: first-layer neurons of the sparsified MLP (later layers need the whole first layer)
    c = workloads.cfg5()
    ct = keys.encrypt(c["x"], c["enc_seed"])
    L1 = c["layers"][0]
    plain = cc.dense_plain(c["x"], L1["W"], L1["T"])
    for j in CFG5_L1_NEURONS:
        if known("cfg5", [0, j]):
            continue
        cir, outs = cc.dense_layer(784, L1["W"][j:j + 1], L1["T"][j:j + 1])
        res, _ = cc.eval_encrypted(keys, cir, ct, outs, threads)
        record("cfg5", [0, j], res[0], plain[j], len(cir.gates))

    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
