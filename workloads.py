"""Seeded synthetic inputs: the five benchmark configurations, and whole networks in the
shapes of the paper's own models.

This module holds no arithmetic of the method: it only draws bits, weights and
thresholds with numpy's seeded generator.  The oracle-side tests and the GPU-side
tests / benchmark both take their inputs from here so that they see the same data.

The shapes follow the workloads of the TAPAS paper where they coincide (Sec. 5.2:
a 28x28 binary image = 784 bits; convolutions with 32 output channels and unit
stride); the paper's datasets and trained weights are not used.
"""
import numpy as np

MASTER = 180603461 * 16
KEY_SEED = 0x7A9A5EED


def seed_of(cfg):
    return MASTER + cfg


def _rng(cfg, sub=0):
    return np.random.Generator(np.random.PCG64([seed_of(cfg), sub]))


def cfg1():
    """16 independent gates: 8 NAND then 8 XNOR on uniform bits."""
    r = _rng(1)
    a = r.integers(0, 2, 16).astype(np.uint8)
    b = r.integers(0, 2, 16).astype(np.uint8)
    ops = ["NAND"] * 8 + ["XNOR"] * 8
    return {"a": a, "b": b, "ops": ops, "enc_seed": seed_of(1) * 3 + 1}


def cfg2(T=None):
    """One neuron, 256 inputs, +-1 weights, integer threshold on the popcount."""
    r = _rng(2)
    x = (r.random(256) < 0.5).astype(np.uint8)
    w = (2 * r.integers(0, 2, 256) - 1).astype(np.int8)
    t = int(r.integers(96, 161)) if T is None else int(T)
    return {"x": x, "W": w.reshape(1, 256), "T": np.array([t], np.int32), "enc_seed": seed_of(2) * 3 + 1}


def cfg3(p=512, d=784):
    """Fully connected layer 784 -> 512, thresholds uniform in [300, 484]."""
    r = _rng(3)
    x = (r.random(d) < 0.5).astype(np.uint8)
    W = (2 * r.integers(0, 2, (p, d)) - 1).astype(np.int8)
    T = r.integers(300, 485, p).astype(np.int32)
    return {"x": x, "W": W, "T": T, "enc_seed": seed_of(3) * 3 + 1}


def cfg4(C=16, H=28, Wd=28, O=32):
    """3x3 convolution, stride 1, pad 1, 16 -> 32 channels on 28x28 bits."""
    r = _rng(4)
    x = (r.random((C, H, Wd)) < 0.5).astype(np.uint8)
    K = (2 * r.integers(0, 2, (O, C, 3, 3)) - 1).astype(np.int8)
    T = r.integers(55, 90, O).astype(np.int32)
    return {"x": x, "K": K, "T": T, "stride": 1, "pad": 1, "enc_seed": seed_of(4) * 3 + 1}


def cfg5(sizes=(784, 256, 256, 10)):
    """Sparsified MLP: +-1 weights, half of them zeroed; hidden thresholds in
    [ceil(0.38 m), floor(0.62 m)] for a row with m non-zero weights; the last layer
    has no threshold (its popcounts are the scores)."""
    r = _rng(5)
    x = (r.random(sizes[0]) < 0.5).astype(np.uint8)
    layers = []
    for li in range(len(sizes) - 1):
        d, p = sizes[li], sizes[li + 1]
        W = (2 * r.integers(0, 2, (p, d)) - 1).astype(np.int8)
        W[r.random((p, d)) < 0.5] = 0
        m = (W != 0).sum(axis=1)
        if li < len(sizes) - 2:
            lo = np.ceil(0.38 * m).astype(np.int64)
            hi = np.floor(0.62 * m).astype(np.int64)
            T = (lo + (r.random(p) * (hi - lo + 1)).astype(np.int64)).astype(np.int32)
        else:
            T = None
        layers.append({"W": W, "T": T})
    return {"x": x, "layers": layers, "out_bits": 10, "enc_seed": seed_of(5) * 3 + 1}


# ---- networks in the shapes of the paper's own models (Sec. 5.2) ------------------------------
# Only the shapes are the paper's; inputs, weights and thresholds are drawn here.  A hidden
# layer's batch normalisation and sign are one integer threshold per unit, drawn uniformly in
# [ceil(0.4 m), floor(0.6 m)] for fan-in m; a network's last layer has no threshold and emits
# its popcounts (the batch normalisation after it is the client's affine map on the decrypted
# scores).

def _thresholds(r, count, m):
    lo, hi = int(np.ceil(0.4 * m)), int(np.floor(0.6 * m))
    return r.integers(lo, hi + 1, count).astype(np.int32)


def paper_cancer():
    """One fully connected layer 90 -> 1 on a 90-bit one-hot-binned record; the score is the
    7-bit popcount."""
    r = _rng(11)
    x = (r.random(90) < 1.0 / 3.0).astype(np.uint8)        # one of three bins per feature
    W = (2 * r.integers(0, 2, (1, 90)) - 1).astype(np.int8)
    return {"x": x, "layers": [{"W": W, "T": None}], "out_bits": 7, "enc_seed": seed_of(11) * 3 + 1}


def paper_diabetes():
    """Fully connected 1704 -> 10 with sign, then 10 -> 3 scores (4-bit popcounts)."""
    r = _rng(12)
    x = (r.random(1704) < 0.25).astype(np.uint8)
    W1 = (2 * r.integers(0, 2, (10, 1704)) - 1).astype(np.int8)
    W2 = (2 * r.integers(0, 2, (3, 10)) - 1).astype(np.int8)
    return {"x": x, "layers": [{"W": W1, "T": _thresholds(r, 10, 1704)}, {"W": W2, "T": None}],
            "out_bits": 4, "enc_seed": seed_of(12) * 3 + 1}


def paper_faces(channels=32, size=50, window=10):
    """Five convolutions (window x window, unit stride, no padding) on a size x size binary image,
    `channels` output channels each but the last, which has one; then a fully connected layer on
    the flattened map emitting one popcount score.  channels=32, size=50, window=10 is the
    paper's shape (50 -> 41 -> 32 -> 23 -> 14 -> 5, then 25 -> 1); smaller values give the same
    structure at a cost a test can afford.  Every convolution is followed by a threshold here
    (the paper leaves the fifth without activation, which would feed integers, not bits, to
    the last layer)."""
    r = _rng(13)
    x = (r.random((1, size, size)) < 0.5).astype(np.uint8)
    convs, cin, side = [], 1, size
    for li in range(5):
        cout = channels if li < 4 else 1
        K = (2 * r.integers(0, 2, (cout, cin, window, window)) - 1).astype(np.int8)
        convs.append({"K": K, "T": _thresholds(r, cout, cin * window * window), "stride": 1, "pad": 0})
        cin, side = cout, side - window + 1
        assert side >= 1, "image too small for five windows"
    d = cin * side * side
    W = (2 * r.integers(0, 2, (1, d)) - 1).astype(np.int8)
    return {"x": x, "convs": convs, "dense": {"W": W, "T": None}, "out_bits": max(1, int(d).bit_length()),
            "enc_seed": seed_of(13) * 3 + 1}
