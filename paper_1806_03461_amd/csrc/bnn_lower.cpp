// Lowering of binary-neural-network layers to gate circuits, and the layer entry points.
//
// A unit computes z = sign(w.x + b) (TAPAS, Sec. 3.2): XNOR each input with its weight bit,
// count the ones (S), test 2S >= d - b.  With plaintext weights the XNOR is a copy or a
// negation of the input ciphertext (Sec. 4.1.1) and costs nothing: it becomes the sign flag of
// the first gate that consumes the input.  Zero weights drop the input (Sec. 4.3).  The count
// is the reduce tree of half adders and ripple-carry adders of Sec. 4.1.1; the comparison with
// the plaintext threshold is the least-to-most-significant chain of Algorithm 1, each
// multiplexer specialised by its known threshold bit (MUX(s,1,o) = OR, MUX(s,o,0) = AND) and
// started from "equal so far counts as true" so that the result is S >= T.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <new>
#include <thread>

#include "common.h"
#include "kernels.h"

namespace tfhe {
int run_layer_stream(tfhe_cloud_key *ck, const tfhe_gate_rec *gates, size_t ngates, size_t nwires, size_t n_fixed,
                     std::vector<tfhe_out_ref> &outs, hipStream_t stream,
                     const std::function<int(size_t pool_wires, uint32_t **wires)> &prepare);
int ensure_uploaded(tfhe_cloud_key *ck);
}

namespace {

using tfhe::set_error;

// A signal: a wire with an optional negation, or a known constant.
struct Sig {
    int32_t wire;   // -1: constant
    int32_t flag;   // wire: negated?  constant: its value
    static Sig of(int32_t w, bool neg = false) { return Sig{w, neg ? 1 : 0}; }
    static Sig constant(int v) { return Sig{-1, v}; }
    bool is_const() const { return wire < 0; }
};

// A little-endian unsigned number of signals with a known upper bound.
struct Number {
    std::vector<Sig> bits;
    int64_t bound = 0;
};

// wire numbers are int32: a circuit that would need more is refused before any record is handed out
using WireOverflow = tfhe::CircuitTooLarge;

class Builder {
public:
    explicit Builder(int32_t n_inputs, bool share = false)
        : next_(n_inputs + 2), zero_(n_inputs), one_(n_inputs + 1), share_(share) {}
    int32_t zero_wire() const { return zero_; }
    int32_t wires() const { return next_; }
    std::vector<tfhe_gate_rec> &gates() { return gates_; }

    Sig emit(int op, Sig a, Sig b) {
        if (share_) {
            // same opcode on the same unordered pair of literals: reuse the earlier gate's wire
            const uint64_t la = ((uint64_t)(uint32_t)a.wire << 1) | (uint64_t)a.flag;   // < 2^32
            const uint64_t lb = ((uint64_t)(uint32_t)b.wire << 1) | (uint64_t)b.flag;
            int32_t &slot = known_.slot(op, (std::min(la, lb) << 32) | std::max(la, lb));
            if (slot >= 0) return Sig::of(slot);
            slot = next_;
        }
        tfhe_gate_rec r{};
        r.op = (uint8_t)op; r.neg0 = (uint8_t)a.flag; r.neg1 = (uint8_t)b.flag;
        r.in0 = a.wire; r.in1 = b.wire; r.out = take_wire();
        gates_.push_back(r);
        return Sig::of(r.out);
    }

    // sel ? a : b as the two-record multiplexer
    Sig emit_mux(Sig sel, Sig a, Sig b) {
        tfhe_gate_rec r{};
        r.op = TFHE_MUX; r.neg0 = (uint8_t)sel.flag; r.neg1 = (uint8_t)a.flag;
        r.in0 = sel.wire; r.in1 = a.wire; r.out = take_wire();
        gates_.push_back(r);
        r.op = TFHE_MUX_ELSE; r.neg1 = (uint8_t)b.flag; r.in1 = b.wire;
        gates_.push_back(r);
        return Sig::of(r.out);
    }

    // Appending the gates of builders over the same inputs, with their gate wires renumbered,
    // gives what emitting those gates here would have given.  grow() makes room for a part's
    // records and wires and says where they go; place() copies the part there and renumbers its
    // output references `part_outs` (calls for different parts may run concurrently).
    struct Slot { size_t gate_at; int32_t wire_shift; };
    Slot grow(const Builder &part) {
        const Slot s{gates_.size(), next_ - (zero_ + 2)};
        if ((int64_t)next_ + (part.next_ - (zero_ + 2)) > (int64_t)INT32_MAX) throw WireOverflow();
        gates_.resize(gates_.size() + part.gates_.size());
        next_ += part.next_ - (zero_ + 2);
        return s;
    }
    void place(const Builder &part, std::vector<tfhe_out_ref> &part_outs, Slot s) {
        const int32_t first = zero_ + 2;
        tfhe_gate_rec *dst = gates_.data() + s.gate_at;
        for (size_t g = 0; g < part.gates_.size(); ++g) {
            tfhe_gate_rec r = part.gates_[g];
            if (r.in0 >= first) r.in0 += s.wire_shift;
            if (r.in1 >= first) r.in1 += s.wire_shift;
            r.out += s.wire_shift;
            dst[g] = r;
        }
        for (tfhe_out_ref &o : part_outs)
            if (o.wire >= first) o.wire += s.wire_shift;
    }

    static int width_of(int64_t bound) { int w = 0; while (bound >> w) ++w; return w; }

    // Ripple-carry addition; carries are produced only where the bounds allow one.
    Number add(const Number &p, const Number &q) {
        const Number &longer = q.bits.size() > p.bits.size() ? q : p;
        const Number &shorter = q.bits.size() > p.bits.size() ? p : q;
        Number sum;
        sum.bound = p.bound + q.bound;
        const int width = width_of(sum.bound);
        const int nl = (int)longer.bits.size(), ns = (int)shorter.bits.size();
        Sig carry = Sig::constant(0);
        bool have_carry = false;
        for (int pos = 0; pos < nl; ++pos) {
            const bool wants_carry = pos + 1 < width;
            const Sig x = longer.bits[pos];
            if (pos == 0) {                                   // half adder
                const Sig y = shorter.bits[0];
                sum.bits.push_back(emit(TFHE_XOR, x, y));
                if (wants_carry) { carry = emit(TFHE_AND, x, y); have_carry = true; }
            } else if (pos < ns) {                            // full adder
                const Sig y = shorter.bits[pos];
                const Sig t = emit(TFHE_XOR, x, y);
                sum.bits.push_back(emit(TFHE_XOR, t, carry));
                if (wants_carry) {
                    const Sig gen = emit(TFHE_AND, x, y);
                    const Sig prop = emit(TFHE_AND, t, carry);
                    carry = emit(TFHE_OR, gen, prop);
                }
            } else {                                          // half adder on the carry
                sum.bits.push_back(emit(TFHE_XOR, x, carry));
                if (wants_carry) carry = emit(TFHE_AND, x, carry);
            }
        }
        if (width > nl && have_carry) sum.bits.push_back(carry);
        return sum;
    }

    Number popcount(const std::vector<Sig> &leaves) {
        std::vector<Number> level;
        level.reserve(leaves.size());
        for (const Sig &s : leaves) { Number one; one.bits.push_back(s); one.bound = 1; level.push_back(std::move(one)); }
        if (level.empty()) return Number{};
        while (level.size() > 1) {
            std::vector<Number> next;
            next.reserve(level.size() / 2 + 1);
            size_t i = 0;
            for (; i + 1 < level.size(); i += 2) next.push_back(add(level[i], level[i + 1]));
            if (i < level.size()) next.push_back(std::move(level[i]));
            level.swap(next);
        }
        return std::move(level[0]);
    }

    // [S >= T]
    Sig at_least(const Number &S, int64_t T) {
        if (T <= 0) return Sig::constant(1);
        if (T > S.bound) return Sig::constant(0);
        bool undecided_true = true;          // nothing but "equal so far" seen: result is the constant 1
        Sig o = Sig::constant(1);
        for (size_t pos = 0; pos < S.bits.size(); ++pos) {
            const bool tbit = (T >> pos) & 1;
            if (undecided_true) {
                if (tbit) { o = S.bits[pos]; undecided_true = false; }
            } else {
                o = emit(tbit ? TFHE_AND : TFHE_OR, S.bits[pos], o);
            }
        }
        return o;
    }

    // [S >= T] with one multiplexer per bit of S, as Algorithm 1 prints it (started from 1)
    Sig at_least_by_mux(const Number &S, int64_t T) {
        const Sig one = Sig::of(one_), zero = Sig::of(zero_);
        Sig o = one;
        for (size_t pos = 0; pos < S.bits.size(); ++pos)
            o = ((T >> pos) & 1) ? emit_mux(S.bits[pos], o, zero) : emit_mux(S.bits[pos], one, o);
        if (T < 0) return Sig::constant(1);
        if (T >> S.bits.size()) return Sig::constant(0);
        return o;
    }

    // 2^w - 1 - S: every bit negated, no gate
    static Number complement(const Number &S) {
        Number c;
        c.bits = S.bits;
        for (Sig &b : c.bits) b.flag ^= 1;
        c.bound = ((int64_t)1 << S.bits.size()) - 1;
        return c;
    }

    // The "+1" trick: [S >= T] from a tree over the rarer weight sign and the shared popcount X
    // of all inputs.  2P - X >= c  <=>  2P + ~X >= c + (2^wx - 1);  X - 2Q >= c  <=>
    // X + 2(~Q) >= c + 2(2^wq - 1);  c = T - |neg|.  Bit 0 of the sum is bit 0 of the unshifted
    // operand, the rest is one ripple-carry addition.
    Sig at_least_plus_one(const std::vector<Sig> &inputs, const int8_t *w, int64_t T, const Number &X) {
        std::vector<Sig> pos, neg;
        for (size_t i = 0; i < inputs.size(); ++i) (w[i] > 0 ? pos : neg).push_back(inputs[i]);
        const int64_t c = T - (int64_t)neg.size();
        Number small, other;
        int64_t offset;
        if (pos.size() <= neg.size()) {
            small = popcount(pos);
            other = complement(X);
            offset = other.bound;
        } else {
            small = complement(popcount(neg));
            other = X;
            offset = 2 * small.bound;
        }
        Number high;
        high.bits.assign(other.bits.begin() + 1, other.bits.end());
        high.bound = other.bound >> 1;
        Number total;
        if (!small.bits.empty() && !high.bits.empty()) total = add(small, high);
        else total = small.bits.empty() ? high : small;
        Number U;
        U.bits.push_back(other.bits[0]);
        U.bits.insert(U.bits.end(), total.bits.begin(), total.bits.end());
        U.bound = 2 * total.bound + 1;
        return at_least(U, c + offset);
    }

    // [at least T of the leaves are 1] as position T-1 of a descending bitonic sort
    Sig at_least_by_sorting(const std::vector<Sig> &leaves, int64_t T) {
        const size_t m = leaves.size();
        if (T <= 0) return Sig::constant(1);
        if (T > (int64_t)m) return Sig::constant(0);
        size_t n = 1;
        while (n < m) n *= 2;
        // network entries: a literal, a known zero, or the output of a local (not yet emitted) gate
        struct Entry { int kind; Sig lit; int32_t gate; };     // kind 0 literal, 1 zero, 2 local gate
        struct Local { int op; Entry x, y; };
        std::vector<Entry> a(n, Entry{1, Sig::constant(0), -1});
        for (size_t i = 0; i < m; ++i) a[i] = Entry{0, leaves[i], -1};
        std::vector<Local> local;
        auto swap_pair = [&](size_t i, size_t l) {
            const Entry x = a[i], y = a[l];
            if (y.kind == 1) return;
            if (x.kind == 1) { a[i] = y; a[l] = x; return; }
            local.push_back(Local{TFHE_OR, x, y});
            local.push_back(Local{TFHE_AND, x, y});
            a[i] = Entry{2, Sig::constant(0), (int32_t)local.size() - 2};
            a[l] = Entry{2, Sig::constant(0), (int32_t)local.size() - 1};
        };
        for (size_t k = 2; k <= n; k *= 2) {
            for (size_t i = 0; i < n; ++i) { const size_t l = i ^ (k - 1); if (l > i) swap_pair(i, l); }
            for (size_t j = k / 4; j >= 1; j /= 2)
                for (size_t i = 0; i < n; ++i) { const size_t l = i ^ j; if (l > i) swap_pair(i, l); }
        }
        const Entry out = a[(size_t)T - 1];
        if (out.kind == 0) return out.lit;
        // keep the cone of the selected position only, emit it in network order
        std::vector<char> needed(local.size(), 0);
        std::vector<int32_t> stack{out.gate};
        while (!stack.empty()) {
            const int32_t g = stack.back();
            stack.pop_back();
            if (needed[g]) continue;
            needed[g] = 1;
            if (local[g].x.kind == 2) stack.push_back(local[g].x.gate);
            if (local[g].y.kind == 2) stack.push_back(local[g].y.gate);
        }
        std::vector<Sig> wire(local.size(), Sig::constant(0));
        for (size_t g = 0; g < local.size(); ++g) {
            if (!needed[g]) continue;
            const Sig lx = local[g].x.kind == 0 ? local[g].x.lit : wire[local[g].x.gate];
            const Sig ly = local[g].y.kind == 0 ? local[g].y.lit : wire[local[g].y.gate];
            wire[g] = emit(local[g].op, lx, ly);
        }
        return wire[out.gate];
    }

    // one output unit over the listed inputs
    void unit(const std::vector<Sig> &inputs, const int8_t *w, const int32_t *T, int out_bits,
              std::vector<tfhe_out_ref> &outs, uint32_t flags = 0) {
        std::vector<Sig> leaves;
        leaves.reserve(inputs.size());
        for (size_t i = 0; i < inputs.size(); ++i) {
            if (w[i] == 0) continue;
            Sig s = inputs[i];
            if (w[i] < 0) s.flag ^= 1;
            leaves.push_back(s);
        }
        if (T && (flags & TFHE_LOWER_SORTING_NETWORK)) {
            const Sig o = at_least_by_sorting(leaves, *T);
            outs.push_back(tfhe_out_ref{o.wire, o.flag});
            return;
        }
        const Number S = popcount(leaves);
        if (T) {
            const Sig o = (flags & TFHE_LOWER_MUX_COMPARATOR) ? at_least_by_mux(S, *T) : at_least(S, *T);
            outs.push_back(tfhe_out_ref{o.wire, o.flag});
        } else {
            for (int bpos = 0; bpos < out_bits; ++bpos) {
                if (bpos < (int)S.bits.size()) outs.push_back(tfhe_out_ref{S.bits[bpos].wire, S.bits[bpos].flag});
                else outs.push_back(tfhe_out_ref{-1, 0});
            }
        }
    }

private:
    int32_t take_wire() {
        if (next_ == INT32_MAX) throw WireOverflow();
        return next_++;
    }
    std::vector<tfhe_gate_rec> gates_;
    int32_t next_, zero_, one_;
    bool share_;

    // open-addressing table (opcode, literal pair) -> wire; grows by doubling
    struct GateTable {
        std::vector<uint64_t> keys;
        std::vector<int32_t> wires;      // -1 = empty slot
        std::vector<uint8_t> ops;
        size_t used = 0;
        static size_t mix(uint64_t k, int op) {
            k ^= (uint64_t)op * 0x9E3779B97F4A7C15ull;
            k ^= k >> 32; k *= 0xD6E8FEB86659FD93ull; k ^= k >> 32;
            return (size_t)k;
        }
        void grow() {
            GateTable bigger;
            const size_t cap = keys.empty() ? (size_t)1 << 16 : keys.size() * 2;
            bigger.keys.assign(cap, 0); bigger.wires.assign(cap, -1); bigger.ops.assign(cap, 0);
            for (size_t i = 0; i < keys.size(); ++i)
                if (wires[i] >= 0) bigger.slot(ops[i], keys[i]) = wires[i];
            bigger.used = used;
            *this = std::move(bigger);
        }
        // the slot of (op, key): its wire if present, else an empty slot (value -1) to fill
        int32_t &slot(int op, uint64_t key) {
            if ((used + 1) * 10 >= keys.size() * 7) grow();
            const size_t mask = keys.size() - 1;
            for (size_t at = mix(key, op) & mask;; at = (at + 1) & mask) {
                if (wires[at] < 0) { keys[at] = key; ops[at] = (uint8_t)op; ++used; return wires[at]; }
                if (keys[at] == key && ops[at] == op) return wires[at];
            }
        }
    } known_;
};

template <class T>
int hand_over(const std::vector<T> &v, T **out, size_t *count) {
    *count = v.size();
    *out = (T *)malloc(std::max<size_t>(1, v.size()) * sizeof(T));
    if (!*out) return set_error(TFHE_E_ALLOC, "out of memory");
    if (!v.empty()) memcpy(*out, v.data(), v.size() * sizeof(T));
    return TFHE_OK;
}

int check_weights(const int8_t *W, size_t count) {
    for (size_t i = 0; i < count; ++i)
        if (W[i] < -1 || W[i] > 1) return set_error(TFHE_E_PARAM, "weight %zu is %d, not in {-1,0,1}", i, W[i]);
    return TFHE_OK;
}

// Units that share nothing are lowered by several host threads, each into a builder of its own
// over a contiguous range of units; appending the parts in order gives exactly the records and
// wire numbers of the serial loop.  per_unit(builder, outs, j) lowers unit j.  Four threads: the
// work is allocation-bound and does not scale further (cfg 3 layer: 234 ms on one thread, 104 ms
// on four, 158 ms on eight).
template <class PerUnit>
int lower_units(int count, size_t work_per_unit, int32_t n_inputs, Builder &b, std::vector<tfhe_out_ref> &outs,
                PerUnit per_unit) {
    int threads = (int)std::min<size_t>(std::min<unsigned>(4u, std::max(1u, std::thread::hardware_concurrency())),
                                        (size_t)count);
    if ((size_t)count * work_per_unit < 200000) threads = 1;
    if (const char *e = getenv("TFHE_LOWER_THREADS")) {           // measurement and tests
        const int v = atoi(e);
        if (v >= 1) threads = std::min(v, count);
    }
    if (threads <= 1) {
        for (int j = 0; j < count; ++j) per_unit(b, outs, j);
        return TFHE_OK;
    }
    struct Part {
        Builder b;
        std::vector<tfhe_out_ref> outs;
        bool failed = false, overflow = false;
        explicit Part(int32_t n) : b(n) {}
    };
    std::vector<Part> parts;
    parts.reserve(threads);
    for (int t = 0; t < threads; ++t) parts.emplace_back(n_inputs);
    std::vector<std::thread> pool;
    for (int t = 0; t < threads; ++t)
        pool.emplace_back([&, t]() {
            const int lo = (int)((int64_t)count * t / threads), hi = (int)((int64_t)count * (t + 1) / threads);
            try {
                // about 7 gate records per input of a reduce-tree unit
                parts[t].b.gates().reserve((size_t)(hi - lo) * work_per_unit * 7 + 64);
                for (int j = lo; j < hi; ++j) per_unit(parts[t].b, parts[t].outs, j);
            } catch (const WireOverflow &) {
                parts[t].overflow = true;
            } catch (...) {
                parts[t].failed = true;
            }
        });
    for (std::thread &th : pool) th.join();
    for (Part &part : parts) {
        if (part.overflow) throw WireOverflow();
        if (part.failed) return set_error(TFHE_E_ALLOC, "out of host memory while lowering");
    }
    std::vector<Builder::Slot> slots;
    for (Part &part : parts) slots.push_back(b.grow(part.b));
    pool.clear();
    for (int t = 0; t < threads; ++t) pool.emplace_back([&, t]() { b.place(parts[t].b, parts[t].outs, slots[t]); });
    for (std::thread &th : pool) th.join();
    for (Part &part : parts) outs.insert(outs.end(), part.outs.begin(), part.outs.end());
    return TFHE_OK;
}

int lower_dense(int d, const int8_t *W, const int32_t *T, int p, int out_bits, uint32_t flags, Builder &b,
                std::vector<tfhe_out_ref> &outs) {
    if (flags & ~(uint32_t)(TFHE_LOWER_MUX_COMPARATOR | TFHE_LOWER_PLUS_ONE | TFHE_LOWER_SHARE_GATES |
                            TFHE_LOWER_SORTING_NETWORK))
        return set_error(TFHE_E_PARAM, "unknown lowering flags %u", flags);
    if ((flags & TFHE_LOWER_SORTING_NETWORK) && (flags & (TFHE_LOWER_MUX_COMPARATOR | TFHE_LOWER_PLUS_ONE)))
        return set_error(TFHE_E_PARAM, "the sorting network excludes the MUX comparator and the +1 trick");
    if (d < 1 || p < 1) return set_error(TFHE_E_SIZE, "layer sizes must be positive");
    if (!W) return set_error(TFHE_E_NULL, "W is NULL");
    if (!T) {
        if (out_bits < 1 || out_bits > 31) return set_error(TFHE_E_SIZE, "out_bits must be in [1,31]");
        int64_t most = 0;
        for (int j = 0; j < p; ++j) {
            int64_t m = 0;
            for (int i = 0; i < d; ++i) m += W[(size_t)j * d + i] != 0;
            most = std::max(most, m);
        }
        if (Builder::width_of(most) > out_bits)
            return set_error(TFHE_E_SIZE, "out_bits=%d cannot hold a popcount of %lld", out_bits, (long long)most);
    }
    if (int rc = check_weights(W, (size_t)d * p)) return rc;
    std::vector<Sig> x(d);
    for (int i = 0; i < d; ++i) x[i] = Sig::of(i);
    if (!(flags & (TFHE_LOWER_PLUS_ONE | TFHE_LOWER_SHARE_GATES)))
        return lower_units(p, (size_t)d, d, b, outs, [&](Builder &bb, std::vector<tfhe_out_ref> &oo, int j) {
            bb.unit(x, W + (size_t)j * d, T ? T + j : nullptr, out_bits, oo, flags);
        });
    Number X;          // popcount of all inputs, built on first use, shared by the layer's units
    for (int j = 0; j < p; ++j) {
        const int8_t *w = W + (size_t)j * d;
        const bool dense_row = std::all_of(w, w + d, [](int8_t v) { return v != 0; });
        if ((flags & TFHE_LOWER_PLUS_ONE) && T && d > 1 && dense_row) {
            if (X.bits.empty()) X = b.popcount(x);
            const Sig o = b.at_least_plus_one(x, w, T[j], X);
            outs.push_back(tfhe_out_ref{o.wire, o.flag});
        } else {
            b.unit(x, w, T ? T + j : nullptr, out_bits, outs, flags);
        }
    }
    return TFHE_OK;
}

// Units u0 <= u < u1 of the convolution in output order (u = (o * Ho + y) * Wo + x); a range other
// than all units is only possible where units are lowered independently of each other.
int lower_conv(int C, int H, int Wd, const int8_t *K, int O, int kh, int kw, int stride, int pad,
               const int32_t *T, uint32_t flags, Builder &b, std::vector<tfhe_out_ref> &outs,
               long long u0 = 0, long long u1 = -1) {
    if (flags & ~(uint32_t)(TFHE_LOWER_PLUS_ONE | TFHE_LOWER_SHARE_GATES | TFHE_LOWER_SORTING_NETWORK))
        return set_error(TFHE_E_PARAM, "unknown lowering flags %u", flags);
    if ((flags & TFHE_LOWER_SORTING_NETWORK) && (flags & TFHE_LOWER_PLUS_ONE))
        return set_error(TFHE_E_PARAM, "the sorting network excludes the +1 trick");
    if (C < 1 || H < 1 || Wd < 1 || O < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0)
        return set_error(TFHE_E_SIZE, "bad convolution shape");
    if (!K || !T) return set_error(TFHE_E_NULL, "K or T is NULL");
    if (H + 2 * pad < kh || Wd + 2 * pad < kw) return set_error(TFHE_E_SIZE, "kernel larger than padded image");
    const size_t taps = (size_t)C * kh * kw;
    if (int rc = check_weights(K, taps * O)) return rc;
    const int Ho = (H + 2 * pad - kh) / stride + 1, Wo = (Wd + 2 * pad - kw) / stride + 1;
    auto gather_field = [=](std::vector<Sig> &f, int y, int x, int32_t zero_wire) {
        size_t t = 0;
        for (int c = 0; c < C; ++c)
            for (int ky = 0; ky < kh; ++ky)
                for (int kx = 0; kx < kw; ++kx, ++t) {
                    const int iy = y * stride + ky - pad, ix = x * stride + kx - pad;
                    const bool inside = iy >= 0 && iy < H && ix >= 0 && ix < Wd;
                    f[t] = Sig::of(inside ? (c * H + iy) * Wd + ix : zero_wire);
                }
    };
    if (!(flags & (TFHE_LOWER_PLUS_ONE | TFHE_LOWER_SHARE_GATES))) {
        if ((long long)O * Ho * Wo > INT32_MAX) return set_error(TFHE_E_SIZE, "too many output pixels");
        if (u1 < 0) u1 = (long long)O * Ho * Wo;
        return lower_units((int)(u1 - u0), taps, C * H * Wd, b, outs,
                           [&](Builder &bb, std::vector<tfhe_out_ref> &oo, int k) {
                               thread_local std::vector<Sig> f;
                               f.resize(taps);
                               const int u = (int)u0 + k;
                               const int o = u / (Ho * Wo), y = u / Wo % Ho, x = u % Wo;
                               gather_field(f, y, x, bb.zero_wire());
                               bb.unit(f, K + (size_t)o * taps, T + o, 0, oo, flags);
                           });
    }
    std::vector<Sig> field(taps);
    // "+1" trick: the popcount of a pixel's receptive field is shared by its output channels
    std::vector<Number> field_sum((flags & TFHE_LOWER_PLUS_ONE) ? (size_t)Ho * Wo : 0);
    for (int o = 0; o < O; ++o)
        for (int y = 0; y < Ho; ++y)
            for (int x = 0; x < Wo; ++x) {
                gather_field(field, y, x, b.zero_wire());
                const int8_t *w = K + (size_t)o * taps;
                const bool dense_row = std::all_of(w, w + taps, [](int8_t v) { return v != 0; });
                if ((flags & TFHE_LOWER_PLUS_ONE) && taps > 1 && dense_row) {
                    Number &X = field_sum[(size_t)y * Wo + x];
                    if (X.bits.empty()) X = b.popcount(field);
                    const Sig s = b.at_least_plus_one(field, w, T[o], X);
                    outs.push_back(tfhe_out_ref{s.wire, s.flag});
                } else {
                    b.unit(field, w, T + o, 0, outs, flags);
                }
            }
    return TFHE_OK;
}

// A layer whose units are lowered independently of each other is evaluated in groups of units
// when its circuit is large: the host then never holds more than one group's records, and the
// wire pool never more than one group's live wires, whatever the layer's size.  The bound is on
// the estimated gates of a group; the function returns the units per group.
long long units_per_group(long long units, size_t inputs_per_unit, uint32_t flags) {
    if (flags & (TFHE_LOWER_PLUS_ONE | TFHE_LOWER_SHARE_GATES)) return units;     // units share gates
    long long budget = 48ll << 20;                                                  // gates per group
    if (const char *e = getenv("TFHE_LAYER_GROUP_GATES")) {                        // measurement and tests
        const long long v = atoll(e);
        if (v > 0) budget = v;
    }
    // gates per input: about 7 for the reduce tree, several times that for the sorting network
    const long long per_unit = (long long)std::max<size_t>(1, inputs_per_unit) * ((flags & TFHE_LOWER_SORTING_NETWORK) ? 48 : 7);
    return std::max<long long>(1, std::min(units, budget / per_unit));
}

// the statistics of a layer call cover all its groups: gates and wires add up, the pool is the largest
struct LayerTotals {
    size_t gates = 0, wires = 0, pool = 0, levels = 0;
    void add(const tfhe_cloud_key *ck) {
        gates += ck->last_layer_gates; wires += ck->last_layer_wires;
        pool = std::max(pool, ck->last_layer_pool); levels = std::max(levels, ck->last_layer_levels);
    }
    void store(tfhe_cloud_key *ck) const {
        ck->last_layer_gates = gates; ck->last_layer_wires = wires; ck->last_layer_pool = pool; ck->last_layer_levels = levels;
    }
};

// wire pool = [inputs | noiseless 0 | noiseless 1 | recycled slots of the gate outputs]; run; gather the outputs
int evaluate(tfhe_cloud_key *ck, Builder &b, std::vector<tfhe_out_ref> &outs, const uint32_t *x,
             int n_inputs, uint32_t *out, hipStream_t stream) {
    const int words = ck->params.n + 1;
    uint32_t *wires = nullptr;
    auto prepare = [&](size_t pool_wires, uint32_t **pool) -> int {
        if (int rc = ck->ws_wires.reserve(pool_wires * words * sizeof(uint32_t))) return rc;
        wires = (uint32_t *)ck->ws_wires.ptr;
        TFHE_HIP(hipMemcpyAsync(wires, x, (size_t)n_inputs * words * sizeof(uint32_t), hipMemcpyDeviceToDevice, stream));
        if (int rc = tfhe::launch_fill_trivial(wires + (size_t)n_inputs * words, words, 0, stream)) return rc;
        if (int rc = tfhe::launch_fill_trivial(wires + (size_t)(n_inputs + 1) * words, words, 1, stream)) return rc;
        *pool = wires;
        return TFHE_OK;
    };
    if (int rc = tfhe::run_layer_stream(ck, b.gates().data(), b.gates().size(), (size_t)b.wires(), (size_t)n_inputs + 2,
                                        outs, stream, prepare))
        return rc;
    if (int rc = ck->ws_outs.reserve(std::max<size_t>(1, outs.size()) * sizeof(tfhe_out_ref))) return rc;
    // the output references go through pinned staging as well: no host wait
    if (int rc = ck->stage_outs.reserve(std::max<size_t>(1, outs.size()) * sizeof(tfhe_out_ref))) return rc;
    if (!outs.empty()) memcpy(ck->stage_outs.ptr, outs.data(), outs.size() * sizeof(tfhe_out_ref));
    TFHE_HIP(hipMemcpyAsync(ck->ws_outs.ptr, ck->stage_outs.ptr, outs.size() * sizeof(tfhe_out_ref),
                            hipMemcpyHostToDevice, stream));
    if (int rc = ck->stage_outs.mark(stream)) return rc;
    return tfhe::launch_gather_outputs(wires, (const tfhe_out_ref *)ck->ws_outs.ptr, out, outs.size(), words, stream);
}

}  // namespace

extern "C" {

int bnn_dense_lower(int d, const int8_t *W, const int32_t *T, int p, int out_bits, tfhe_gate_rec **gates,
                    size_t *ngates, tfhe_out_ref **outs, size_t *nouts, size_t *nwires) {
    return bnn_dense_lower_opts(d, W, T, p, out_bits, TFHE_LOWER_DEFAULT, gates, ngates, outs, nouts, nwires);
}

static int bnn_dense_lower_opts_impl(int d, const int8_t *W, const int32_t *T, int p, int out_bits, uint32_t flags,
                         tfhe_gate_rec **gates, size_t *ngates, tfhe_out_ref **outs, size_t *nouts,
                         size_t *nwires) {
    if (!gates || !ngates || !outs || !nouts || !nwires) return set_error(TFHE_E_NULL, "NULL output pointer");
    if (d < 1) return set_error(TFHE_E_SIZE, "layer sizes must be positive");
    Builder b(d, (flags & TFHE_LOWER_SHARE_GATES) != 0);
    std::vector<tfhe_out_ref> o;
    if (int rc = lower_dense(d, W, T, p, out_bits, flags, b, o)) return rc;
    if (int rc = hand_over(b.gates(), gates, ngates)) return rc;
    if (int rc = hand_over(o, outs, nouts)) { free(*gates); return rc; }
    *nwires = (size_t)b.wires();
    return TFHE_OK;
}

int bnn_dense_lower_opts(int d, const int8_t *W, const int32_t *T, int p, int out_bits, uint32_t flags,
                         tfhe_gate_rec **gates, size_t *ngates, tfhe_out_ref **outs, size_t *nouts,
                         size_t *nwires) {
    return tfhe::guarded([&]() -> int { return bnn_dense_lower_opts_impl(d, W, T, p, out_bits, flags, gates, ngates, outs, nouts, nwires); });
}

int bnn_conv_lower(int C, int H, int Wd, const int8_t *K, int O, int kh, int kw, int stride, int pad,
                   const int32_t *T, tfhe_gate_rec **gates, size_t *ngates, tfhe_out_ref **outs, size_t *nouts,
                   size_t *nwires) {
    return bnn_conv_lower_opts(C, H, Wd, K, O, kh, kw, stride, pad, T, TFHE_LOWER_DEFAULT, gates, ngates, outs,
                               nouts, nwires);
}

static int bnn_conv_lower_opts_impl(int C, int H, int Wd, const int8_t *K, int O, int kh, int kw, int stride, int pad,
                        const int32_t *T, uint32_t flags, tfhe_gate_rec **gates, size_t *ngates,
                        tfhe_out_ref **outs, size_t *nouts, size_t *nwires) {
    if (!gates || !ngates || !outs || !nouts || !nwires) return set_error(TFHE_E_NULL, "NULL output pointer");
    if (C < 1 || H < 1 || Wd < 1 || (long long)C * H * Wd > (1ll << 30))
        return set_error(TFHE_E_SIZE, "bad convolution shape");
    Builder b(C * H * Wd, (flags & TFHE_LOWER_SHARE_GATES) != 0);
    std::vector<tfhe_out_ref> o;
    if (int rc = lower_conv(C, H, Wd, K, O, kh, kw, stride, pad, T, flags, b, o)) return rc;
    if (int rc = hand_over(b.gates(), gates, ngates)) return rc;
    if (int rc = hand_over(o, outs, nouts)) { free(*gates); return rc; }
    *nwires = (size_t)b.wires();
    return TFHE_OK;
}

int bnn_conv_lower_opts(int C, int H, int Wd, const int8_t *K, int O, int kh, int kw, int stride, int pad,
                        const int32_t *T, uint32_t flags, tfhe_gate_rec **gates, size_t *ngates,
                        tfhe_out_ref **outs, size_t *nouts, size_t *nwires) {
    return tfhe::guarded([&]() -> int { return bnn_conv_lower_opts_impl(C, H, Wd, K, O, kh, kw, stride, pad, T, flags, gates, ngates, outs, nouts, nwires); });
}

int bnn_dense_encrypted(tfhe_cloud_key *ck, const uint32_t *x, int d, const int8_t *W, const int32_t *T, int p,
                        uint32_t *out, int out_bits, void *stream) {
    return bnn_dense_encrypted_opts(ck, x, d, W, T, p, out, out_bits, TFHE_LOWER_DEFAULT, stream);
}

static int bnn_dense_encrypted_opts_impl(tfhe_cloud_key *ck, const uint32_t *x, int d, const int8_t *W, const int32_t *T,
                             int p, uint32_t *out, int out_bits, uint32_t flags, void *stream) {
    if (int rc = tfhe::ensure_uploaded(ck)) return rc;
    if (!x || !out) return set_error(TFHE_E_NULL, "NULL ciphertext buffer");
    if (d < 1) return set_error(TFHE_E_SIZE, "layer sizes must be positive");
    if (p < 1) return set_error(TFHE_E_SIZE, "layer sizes must be positive");
    if (!W) return set_error(TFHE_E_NULL, "W is NULL");
    const long long group = units_per_group(p, (size_t)d, flags);
    const size_t words = (size_t)ck->params.n + 1, outs_per_unit = T ? 1 : (size_t)std::max(out_bits, 0);
    LayerTotals totals;
    for (long long u0 = 0; u0 < p; u0 += group) {
        const int count = (int)std::min<long long>(group, p - u0);
        Builder b(d, (flags & TFHE_LOWER_SHARE_GATES) != 0);
        std::vector<tfhe_out_ref> o;
        if (int rc = lower_dense(d, W + (size_t)u0 * d, T ? T + u0 : nullptr, count, out_bits, flags, b, o)) return rc;
        if (int rc = evaluate(ck, b, o, x, d, out + (size_t)u0 * outs_per_unit * words, (hipStream_t)stream)) return rc;
        totals.add(ck);
    }
    totals.store(ck);
    return TFHE_OK;
}

int bnn_dense_encrypted_opts(tfhe_cloud_key *ck, const uint32_t *x, int d, const int8_t *W, const int32_t *T,
                             int p, uint32_t *out, int out_bits, uint32_t flags, void *stream) {
    return tfhe::guarded([&]() -> int { return bnn_dense_encrypted_opts_impl(ck, x, d, W, T, p, out, out_bits, flags, stream); });
}

int bnn_conv_encrypted(tfhe_cloud_key *ck, const uint32_t *x, int C, int H, int Wd, const int8_t *K, int O,
                       int kh, int kw, int stride, int pad, const int32_t *T, uint32_t *out, void *stream) {
    return bnn_conv_encrypted_opts(ck, x, C, H, Wd, K, O, kh, kw, stride, pad, T, out, TFHE_LOWER_DEFAULT, stream);
}

static int bnn_conv_encrypted_opts_impl(tfhe_cloud_key *ck, const uint32_t *x, int C, int H, int Wd, const int8_t *K, int O,
                            int kh, int kw, int stride, int pad, const int32_t *T, uint32_t *out, uint32_t flags,
                            void *stream) {
    if (int rc = tfhe::ensure_uploaded(ck)) return rc;
    if (!x || !out) return set_error(TFHE_E_NULL, "NULL ciphertext buffer");
    if (C < 1 || H < 1 || Wd < 1 || (long long)C * H * Wd > (1ll << 30))
        return set_error(TFHE_E_SIZE, "bad convolution shape");
    if (O < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0 || H + 2 * pad < kh || Wd + 2 * pad < kw)
        return set_error(TFHE_E_SIZE, "bad convolution shape");
    const long long Ho = (H + 2 * pad - kh) / stride + 1, Wo = (Wd + 2 * pad - kw) / stride + 1;
    const long long units = (long long)O * Ho * Wo;
    if (units > INT32_MAX) return set_error(TFHE_E_SIZE, "too many output pixels");
    const long long group = units_per_group(units, (size_t)C * kh * kw, flags);
    const size_t words = (size_t)ck->params.n + 1;
    LayerTotals totals;
    for (long long u0 = 0; u0 < units; u0 += group) {
        const long long u1 = std::min(units, u0 + group);
        Builder b(C * H * Wd, (flags & TFHE_LOWER_SHARE_GATES) != 0);
        std::vector<tfhe_out_ref> o;
        if (int rc = lower_conv(C, H, Wd, K, O, kh, kw, stride, pad, T, flags, b, o, u0, u1)) return rc;
        if (int rc = evaluate(ck, b, o, x, C * H * Wd, out + (size_t)u0 * words, (hipStream_t)stream)) return rc;
        totals.add(ck);
    }
    totals.store(ck);
    return TFHE_OK;
}

int bnn_conv_encrypted_opts(tfhe_cloud_key *ck, const uint32_t *x, int C, int H, int Wd, const int8_t *K, int O,
                            int kh, int kw, int stride, int pad, const int32_t *T, uint32_t *out, uint32_t flags,
                            void *stream) {
    return tfhe::guarded([&]() -> int { return bnn_conv_encrypted_opts_impl(ck, x, C, H, Wd, K, O, kh, kw, stride, pad, T, out, flags, stream); });
}

}  // extern "C"
