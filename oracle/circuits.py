"""Circuit layer of the oracle: BNN layers as Boolean circuits.  TEST INFRASTRUCTURE ONLY.

Follows the TAPAS paper: a layer is z = sign(Wx + b) with sign(0) = +1
(Sec. 3.2 'Technical details'); on bits it is XNOR with the weight, popcount S,
then the test 2S >= d - b (steps 1-4 there).  With the weights in the clear the
XNOR is a copy or a negation of the encrypted input (Sec. 4.1.1), a zero weight
drops the input (Sec. 4.3), the popcount is a reduce tree of half adders and
ripple-carry adders (Sec. 4.1.1 'Reduce tree adder'), and the comparison with the
plaintext threshold is the LSB-to-MSB chain of Algorithm 1 with its multiplexers
specialised by the known threshold bit: MUX(s, 1, o) = OR(s, o) and
MUX(s, o, 0) = AND(s, o).

Everything here is plain Python on small integers; gate records use the same
16-byte layout as the C oracle's batch entry point.
"""
import numpy as np

from .oracle import GATE_DTYPE, OP

CONST0 = "const0"
CONST1 = "const1"


class Circuit:
    """A wire pool and a gate list.  Wires 0..n_inputs-1 are the encrypted inputs,
    wire n_inputs is a noiseless encryption of 0, wire n_inputs+1 of 1, every gate
    appends one wire.  A literal is (wire, neg)."""

    def __init__(self, n_inputs, share=False):
        self.n_inputs = n_inputs
        self.c0 = n_inputs
        self.c1 = n_inputs + 1
        self.n_wires = n_inputs + 2
        self.gates = []
        # share=True: a two-input gate with the same opcode and the same unordered pair of
        # (wire, negation) inputs as an earlier one is not emitted again; its wire is reused
        self.share = share
        self.known = {}

    def gate(self, op, a, b):
        if self.share:
            key = (OP[op],) + tuple(sorted((a, b)))
            if key in self.known:
                return self.known[key]
            self.known[key] = (self.n_wires, 0)
        out = self.n_wires
        self.n_wires += 1
        self.gates.append((OP[op], a[1], b[1], 0, a[0], b[0], out))
        return (out, 0)

    def mux(self, sel, a, b):
        """sel ? a : b as the two-record multiplexer (same selector and output wire)."""
        out = self.n_wires
        self.n_wires += 1
        self.gates.append((OP["MUX"], sel[1], a[1], 0, sel[0], a[0], out))
        self.gates.append((OP["MUX_ELSE"], sel[1], b[1], 0, sel[0], b[0], out))
        return (out, 0)

    def gate_array(self):
        return np.array(self.gates, dtype=GATE_DTYPE)


def bitlen(x):
    return int(x).bit_length()


def add_numbers(cir, a, b):
    """Ripple-carry sum of two little-endian encrypted numbers (bits, max).
    Bit 0 is a half adder (XOR, AND); a full-adder cell is XOR, XOR, AND, AND, OR;
    beyond the shorter operand the cell is a half adder on the carry.  A carry is
    only computed where the plaintext maxima allow one."""
    (abits, amax), (bbits, bmax) = a, b
    if len(bbits) > len(abits):
        abits, bbits = bbits, abits
    wa, wb = len(abits), len(bbits)
    M = amax + bmax
    wout = bitlen(M)
    out = [cir.gate("XOR", abits[0], bbits[0])]
    c = cir.gate("AND", abits[0], bbits[0]) if wout > 1 else None
    for i in range(1, wa):
        need_carry = i + 1 < wout
        if i < wb:
            t = cir.gate("XOR", abits[i], bbits[i])
            out.append(cir.gate("XOR", t, c))
            if need_carry:
                g = cir.gate("AND", abits[i], bbits[i])
                p = cir.gate("AND", t, c)
                c = cir.gate("OR", g, p)
        else:
            out.append(cir.gate("XOR", abits[i], c))
            if need_carry:
                c = cir.gate("AND", abits[i], c)
    if wout > wa:
        out.append(c)
    assert len(out) == wout
    return (out, M)


def popcount_tree(cir, leaves):
    """Reduce tree: add neighbours pairwise, an odd last element moves on unchanged."""
    L = [([lit], 1) for lit in leaves]
    if not L:
        return ([], 0)
    while len(L) > 1:
        nxt = [add_numbers(cir, L[i], L[i + 1]) for i in range(0, len(L) - 1, 2)]
        if len(L) & 1:
            nxt.append(L[-1])
        L = nxt
    return L[0]


def threshold_chain(cir, number, T):
    """[S >= T] for the encrypted number S (Algorithm 1, started at 'equal so far
    counts as true' so that the result is >= as the paper's step 4 requires)."""
    bits, m = number
    if T <= 0:
        return CONST1
    if T > m:
        return CONST0
    o = CONST1
    for i, s in enumerate(bits):
        Ti = (T >> i) & 1
        if o is CONST1:
            if Ti:
                o = s
        elif Ti:
            o = cir.gate("AND", s, o)
        else:
            o = cir.gate("OR", s, o)
    return o


def threshold_chain_mux(cir, number, T):
    """Algorithm 1 as printed: one MUX per bit of S, least significant first,
    o = MUX(S_i, 1, o) for a 0 threshold bit and o = MUX(S_i, o, 0) for a 1 bit, the constants
    being noiseless encryptions.  The printed initial value o = 0 would give S > T; the stated
    output is 2S >= d - b, so the chain starts from o = 1 here as well."""
    bits, m = number
    one, zero = (cir.c1, 0), (cir.c0, 0)
    o = one
    for i, s in enumerate(bits):
        if (T >> i) & 1:
            o = cir.mux(s, o, zero)
        else:
            o = cir.mux(s, one, o)
    if T < 0:
        return CONST1
    if T >> len(bits):
        return CONST0
    return o


def complement(number):
    """2^w - 1 - S for a w-bit encrypted number: negate every bit (no gate)."""
    bits, _ = number
    return ([(w, n ^ 1) for (w, n) in bits], (1 << len(bits)) - 1)


def neuron_plus_one(cir, x_literals, w_row, T, X):
    """The '+1' trick (Sec. 4.2): sum only the inputs of the rarer weight sign and use the
    popcount X of all inputs, shared by every unit reading the same inputs.  With
    P = sum of x over w=+1, Q = sum over w=-1, X = P + Q and the agreements S = P + |neg| - Q:
        S >= T  <=>  2P - X >= c  <=>  X - 2Q >= c,      c = T - |neg|.
    The subtraction is an addition of the bitwise complement (negated ciphertexts, free):
        |pos| <= |neg|:  U = 2P + ~X,   test U >= c + (2^wx - 1);
        otherwise:       U = X + 2(~Q), test U >= c + 2 (2^wq - 1).
    The factor 2 is a shift: bit 0 of U is bit 0 of the unshifted operand, the rest is one
    ripple-carry addition.  Weights must be +-1 (a zero weight would change X per unit)."""
    pos = [lit for lit, w in zip(x_literals, w_row) if w > 0]
    neg = [lit for lit, w in zip(x_literals, w_row) if w < 0]
    assert len(pos) + len(neg) == len(x_literals), "the +1 trick needs weights in {-1,+1}"
    c = int(T) - len(neg)
    if len(pos) <= len(neg):
        small = popcount_tree(cir, pos)                    # P
        other = complement(X)                              # ~X
        offset = other[1]
    else:
        small = complement(popcount_tree(cir, neg))        # ~Q
        other = X
        offset = 2 * small[1]
    low = other[0][0]
    high = (other[0][1:], other[1] >> 1)
    if small[0] and high[0]:
        total = add_numbers(cir, small, high)
    else:
        total = small if small[0] else high
    U = ([low] + total[0], 2 * total[1] + 1)
    return [threshold_chain(cir, U, c + offset)]


def sorting_network_unit(cir, leaves, T):
    """[S >= T] by sorting the XNOR bits (Sec. 4.1.1 'Sorting network'): after a descending sort
    the bit at position T-1 is 1 exactly when at least T inputs are 1.  The network is Batcher's
    bitonic sorter on the next power of two (padded with noiseless zeros at the end), every
    compare-exchange SWAP(a, b) = (OR(a, b), AND(a, b)) moving the larger bit to the lower index:
    for block sizes k = 2, 4, ..., n first the pairs (i, i XOR (k-1)), then (i, i XOR j) for
    j = k/4, k/8, ..., 1.  A swap with a known zero needs no gate (OR(a,0) = a, AND(a,0) = 0), and
    only the gates that the selected position depends on are emitted."""
    m = len(leaves)
    if T <= 0:
        return CONST1
    if T > m:
        return CONST0
    n = 1
    while n < m:
        n *= 2
    # local network: entries are ('lit', literal), ('zero',) or ('gate', index into local list)
    a = [("lit", l) for l in leaves] + [("zero",)] * (n - m)
    local = []                                             # (op, entry, entry)

    def swap(i, l):
        x, y = a[i], a[l]
        if y[0] == "zero":
            return
        if x[0] == "zero":
            a[i], a[l] = y, x
            return
        local.append(("OR", x, y))
        local.append(("AND", x, y))
        a[i], a[l] = ("gate", len(local) - 2), ("gate", len(local) - 1)

    k = 2
    while k <= n:
        for i in range(n):
            l = i ^ (k - 1)
            if l > i:
                swap(i, l)
        j = k // 4
        while j >= 1:
            for i in range(n):
                l = i ^ j
                if l > i:
                    swap(i, l)
            j //= 2
        k *= 2
    out = a[T - 1]
    if out[0] == "lit":
        return out[1]
    assert out[0] == "gate"
    needed = [False] * len(local)
    stack = [out[1]]
    while stack:
        g = stack.pop()
        if needed[g]:
            continue
        needed[g] = True
        for e in local[g][1:]:
            if e[0] == "gate":
                stack.append(e[1])
    wire = {}
    for g, (op, x, y) in enumerate(local):
        if needed[g]:
            lx = x[1] if x[0] == "lit" else wire[x[1]]
            ly = y[1] if y[0] == "lit" else wire[y[1]]
            wire[g] = cir.gate(op, lx, ly)
    return wire[out[1]]


def neuron(cir, x_literals, w_row, T, out_bits=0, comparator="folded"):
    """One output unit.  x_literals[i] is the literal of input i; w in {-1,0,+1}.
    Returns one literal/constant (T given) or out_bits popcount literals (T None)."""
    leaves = []
    for lit, w in zip(x_literals, w_row):
        if w > 0:
            leaves.append(lit)
        elif w < 0:
            leaves.append((lit[0], lit[1] ^ 1))
    if T is not None and comparator == "sort":
        return [sorting_network_unit(cir, leaves, int(T))]
    S = popcount_tree(cir, leaves)
    if T is not None:
        if comparator == "mux":
            return [threshold_chain_mux(cir, S, int(T))]
        return [threshold_chain(cir, S, int(T))]
    bits = list(S[0]) + [CONST0] * max(0, out_bits - len(S[0]))
    assert len(bits) == out_bits, "out_bits too small for this popcount"
    return bits


def dense_layer(d, W, T, out_bits=0, comparator="folded", plus_one=False, share=False):
    """Circuit of a fully connected layer.  Returns (circuit, outputs).  With plus_one the rows
    without zero weights use the '+1' trick on one shared popcount of the inputs; with share
    identical gates of different units are emitted once."""
    cir = Circuit(d, share)
    x = [(i, 0) for i in range(d)]
    outs = []
    X = None
    for j in range(W.shape[0]):
        if plus_one and T is not None and d > 1 and (W[j] != 0).all():
            if X is None:
                X = popcount_tree(cir, x)
            outs += neuron_plus_one(cir, x, W[j], T[j], X)
        else:
            outs += neuron(cir, x, W[j], None if T is None else T[j], out_bits, comparator)
    return cir, outs


def conv_pixel_literals(cir, C_, H, Wd, kh, kw, stride, pad, y, x):
    """Receptive field of output pixel (y, x): (c, ky, kx) row-major; a pixel
    outside the image is the noiseless encryption of 0."""
    lits = []
    for c in range(C_):
        for ky in range(kh):
            for kx in range(kw):
                iy, ix = y * stride + ky - pad, x * stride + kx - pad
                if 0 <= iy < H and 0 <= ix < Wd:
                    lits.append(((c * H + iy) * Wd + ix, 0))
                else:
                    lits.append((cir.c0, 0))
    return lits


def conv_layer(C_, H, Wd, K, T, stride, pad, pixels=None, plus_one=False, share=False):
    """Circuit of a convolution layer (or of the listed output pixels (o, y, x) only).  With
    plus_one the popcount of a receptive field is shared by the output channels of its pixel."""
    O, _, kh, kw = K.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (Wd + 2 * pad - kw) // stride + 1
    cir = Circuit(C_ * H * Wd, share)
    if pixels is None:
        pixels = [(o, y, x) for o in range(O) for y in range(Ho) for x in range(Wo)]
    outs = []
    field_sum = {}
    for (o, y, x) in pixels:
        lits = conv_pixel_literals(cir, C_, H, Wd, kh, kw, stride, pad, y, x)
        w = K[o].reshape(-1)
        if plus_one and len(lits) > 1 and (w != 0).all():
            if (y, x) not in field_sum:
                field_sum[(y, x)] = popcount_tree(cir, lits)
            outs += neuron_plus_one(cir, lits, w, T[o], field_sum[(y, x)])
        else:
            outs += neuron(cir, lits, w, T[o])
    return cir, outs


# ---------------------------------------------------------------------------
# plaintext evaluation
# ---------------------------------------------------------------------------
_TRUTH = {OP["NAND"]: lambda a, b: 1 - (a & b), OP["AND"]: lambda a, b: a & b,
          OP["OR"]: lambda a, b: a | b, OP["NOR"]: lambda a, b: 1 - (a | b),
          OP["XOR"]: lambda a, b: a ^ b, OP["XNOR"]: lambda a, b: 1 - (a ^ b)}


def eval_plain(cir, in_bits, outs):
    """Evaluate the circuit on plaintext bits; returns the output bits."""
    w = np.zeros(cir.n_wires, np.uint8)
    w[:cir.n_inputs] = in_bits
    w[cir.c0], w[cir.c1] = 0, 1
    pending = None
    for (op, n0, n1, _, i0, i1, o) in cir.gates:
        if op == OP["MUX"]:
            pending = (int(w[i0]) ^ n0, int(w[i1]) ^ n1)        # selector, value if selected
        elif op == OP["MUX_ELSE"]:
            sel, a = pending
            w[o] = a if sel else int(w[i1]) ^ n1
        else:
            w[o] = _TRUTH[op](int(w[i0]) ^ n0, int(w[i1]) ^ n1)
    res = []
    for lit in outs:
        if lit is CONST0:
            res.append(0)
        elif lit is CONST1:
            res.append(1)
        else:
            res.append(int(w[lit[0]]) ^ lit[1])
    return np.array(res, np.uint8)


def eval_encrypted(keys, cir, in_cts, outs, threads=1):
    """Evaluate the circuit on ciphertexts with the oracle gate; returns (out cts, wires)."""
    n1 = keys.P.n + 1
    wires = np.zeros((cir.n_wires, n1), np.uint32)
    wires[:cir.n_inputs] = in_cts
    wires[cir.c0] = keys.trivial(0)
    wires[cir.c1] = keys.trivial(1)
    if cir.gates:
        keys.run_gates(cir.gate_array(), wires, threads)
    res = np.zeros((len(outs), n1), np.uint32)
    for k, lit in enumerate(outs):
        if lit is CONST0:
            res[k] = keys.trivial(0)
        elif lit is CONST1:
            res[k] = keys.trivial(1)
        else:
            res[k] = wires[lit[0]] if not lit[1] else (0 - wires[lit[0]]).astype(np.uint32)
    return res, wires


# ---------------------------------------------------------------------------
# plaintext BNN layers on integers (Sec. 3.2: z = sign(Wx + b), via popcounts)
# ---------------------------------------------------------------------------
def dense_plain(x_bits, W, T):
    """Bits out: [popcount(XNOR(w, x) over w != 0) >= T]; popcounts if T is None."""
    xs = 2 * x_bits.astype(np.int64) - 1                 # {0,1} -> {-1,+1}
    agree = (W.astype(np.int64) * xs[None, :]) > 0       # XNOR on the +-1 encoding
    S = agree.sum(axis=1)
    if T is None:
        return S
    return (S >= np.asarray(T)).astype(np.uint8)


def conv_plain(x_bits, K, T, stride, pad):
    """x_bits [C,H,W] in {0,1}; padding pixels are bit 0 (i.e. -1), XNORed like any other."""
    C_, H, Wd = x_bits.shape
    O, _, kh, kw = K.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (Wd + 2 * pad - kw) // stride + 1
    xp = np.zeros((C_, H + 2 * pad, Wd + 2 * pad), np.int64)
    xp[:, pad:pad + H, pad:pad + Wd] = x_bits
    xs = 2 * xp - 1
    out = np.zeros((O, Ho, Wo), np.uint8)
    for o in range(O):
        for y in range(Ho):
            for x in range(Wo):
                patch = xs[:, y * stride:y * stride + kh, x * stride:x * stride + kw]
                S = int(((K[o].astype(np.int64) * patch) > 0).sum())
                out[o, y, x] = S >= T[o]
    return out
