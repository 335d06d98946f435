// Host run of the four-wave transform of csrc/fft512.h: the 256 lanes of a workgroup are driven
// one after the other through exactly the per-lane steps the kernels execute (forward, gather,
// products with a transformed key, scatter, inverse), and the rounded results are compared with
// the exact integer negacyclic products  sum_r digit_r * limb_{r,o}  mod X^1024 + 1  computed
// with 64-bit integers.  Operands: random ones and the extremes of the ranges the blind rotation
// feeds (digits in [-512, 511], 16-bit key limbs in [-32768, 32767]), with sign patterns that
// make one coefficient's 4,096 terms add up coherently (|sum| = 2^36, the largest value the
// path must carry).  Prints the largest distance of an unrounded value from an integer.
#include <cinttypes>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../paper_1806_03461_amd/csrc/fft512.h"

using namespace fft512;

namespace {

constexpr int kN = 1024;
typedef std::vector<int64_t> Poly;

std::vector<double2> g_tables(2048);
Lane g_lane[64];
double2 g_buf[kBufWords];
double2 g_x[4][64][8];     // [wave][lane][register]

// the forward half of a step on four polynomials; leaves g_x in gathered order
void forward4(const Poly *const p[4], double scale) {
    for (int w = 0; w < 4; ++w)
        for (int L = 0; L < 64; ++L) {
            for (int m = 0; m < 8; ++m)
                g_x[w][L][m] = make_double2((double)(*p[w])[L + 64 * m] * scale, (double)(*p[w])[L + 64 * m + 512] * scale);
            fwd_pass1_store(g_x[w][L], g_lane[L], g_buf + w * kPolyStride, L);
        }
    // workgroup barrier
    for (int w = 0; w < 4; ++w) {
        for (int L = 0; L < 64; ++L) fwd_pass2_load(g_x[w][L], g_buf + row_of(w, L), L);
        for (int L = 0; L < 64; ++L) fwd_pass2_store(g_x[w][L], g_lane[L], g_buf + row_of(w, L), L);
        for (int L = 0; L < 64; ++L) fwd_pass3(g_x[w][L], g_buf + row_of(w, L), L);
        gather_rows_wave(g_x[w]);
    }
}

// the inverse half on g_x (gathered order); out[o][j] = unrounded coefficient j of polynomial o
void inverse4(std::vector<double> out[4]) {
    for (int w = 0; w < 4; ++w) {
        scatter_rows_wave(g_x[w]);
        for (int L = 0; L < 64; ++L) inv_pass3_store(g_x[w][L], g_lane[L], g_buf + row_of(w, L), L);
        for (int L = 0; L < 64; ++L) inv_pass2(g_x[w][L], g_buf + row_of(w, L), L);
        for (int L = 0; L < 64; ++L) inv_pass2_store(g_x[w][L], g_buf + row_of(w, L), L);
    }
    // workgroup barrier
    for (int o = 0; o < 4; ++o) {
        out[o].assign(kN, 0.0);
        for (int L = 0; L < 64; ++L) {
            inv_pass1(g_x[o][L], g_lane[L], g_buf + o * kPolyStride, L);
            for (int m = 0; m < 8; ++m) {
                out[o][L + 64 * m] = g_x[o][L][m].x;
                out[o][L + 64 * m + 512] = g_x[o][L][m].y;
            }
        }
    }
}

Poly negacyclic(const Poly &a, const Poly &b) {
    Poly c(kN, 0);
    for (int i = 0; i < kN; ++i)
        for (int j = 0; j < kN; ++j) {
            const int k = i + j;
            if (k < kN) c[k] += a[i] * b[j];
            else c[k - kN] -= a[i] * b[j];
        }
    return c;
}

struct Result { long wrong; double worst; };

// one external-product-shaped step: digit[r], limb[r][o] -> sum_r digit[r] * limb[r][o] for o < 4
Result step(const Poly digit[4], const Poly limb[4][4]) {
    // the key in the transform domain, slot order, scaled by 1/512 (what the upload kernel stores)
    static double2 key[4][4][512];
    for (int r = 0; r < 4; ++r) {
        const Poly *four[4] = {&limb[r][0], &limb[r][1], &limb[r][2], &limb[r][3]};
        forward4(four, 1.0 / 512.0);
        for (int w = 0; w < 4; ++w)
            for (int L = 0; L < 64; ++L)
                for (int o = 0; o < 4; ++o)
                    for (int q = 0; q < 2; ++q) key[r][o][256 * q + 64 * w + L] = g_x[w][L][2 * o + q];
    }
    const Poly *four[4] = {&digit[0], &digit[1], &digit[2], &digit[3]};
    forward4(four, 1.0);
    for (int w = 0; w < 4; ++w)
        for (int L = 0; L < 64; ++L) {
            double2 y[8];
            for (int o = 0; o < 4; ++o)
                for (int q = 0; q < 2; ++q) {
                    double2 acc = make_double2(0.0, 0.0);
                    for (int r = 0; r < 4; ++r) acc = cadd(acc, cmul(g_x[w][L][2 * r + q], key[r][o][256 * q + 64 * w + L]));
                    y[2 * o + q] = acc;
                }
            for (int k = 0; k < 8; ++k) g_x[w][L][k] = y[k];
        }
    std::vector<double> got[4];
    inverse4(got);
    Result res{0, 0.0};
    for (int o = 0; o < 4; ++o) {
        Poly want(kN, 0);
        for (int r = 0; r < 4; ++r) {
            const Poly part = negacyclic(digit[r], limb[r][o]);
            for (int j = 0; j < kN; ++j) want[j] += part[j];
        }
        for (int j = 0; j < kN; ++j) {
            const double rounded = nearbyint(got[o][j]);
            if ((int64_t)rounded != want[j]) ++res.wrong;
            res.worst = fmax(res.worst, fabs(got[o][j] - rounded));
        }
    }
    return res;
}

uint64_t g_state = 0x243F6A8885A308D3ull;
uint32_t next_u32() {          // xorshift64*
    g_state ^= g_state >> 12; g_state ^= g_state << 25; g_state ^= g_state >> 27;
    return (uint32_t)((g_state * 0x2545F4914F6CDD1Dull) >> 32);
}

}  // namespace

int main() {
    const long double pi = 3.14159265358979323846264338327950288L;
    for (int j = 0; j < 2048; ++j) g_tables[j] = make_double2((double)cosl(pi * j / 1024), (double)sinl(pi * j / 1024));
    for (int L = 0; L < 64; ++L) lane_init(g_lane[L], g_tables.data(), L);

    long wrong = 0;
    double worst = 0.0;
    auto run = [&](const char *name, const Poly digit[4], const Poly limb[4][4]) {
        const Result r = step(digit, limb);
        printf("%-58s wrong %ld  worst distance %.3g\n", name, r.wrong, r.worst);
        wrong += r.wrong;
        worst = fmax(worst, r.worst);
    };
    Poly digit[4], limb[4][4];
    for (int r = 0; r < 4; ++r) { digit[r].assign(kN, 0); for (int o = 0; o < 4; ++o) limb[r][o].assign(kN, 0); }

    for (int rep = 0; rep < 3; ++rep) {
        for (int r = 0; r < 4; ++r) {
            for (int j = 0; j < kN; ++j) digit[r][j] = (int64_t)(next_u32() % 1024) - 512;
            for (int o = 0; o < 4; ++o)
                for (int j = 0; j < kN; ++j) limb[r][o][j] = (int64_t)(next_u32() % 65536) - 32768;
        }
        run("random digits and limbs", digit, limb);
    }
    // every operand at one end of its range
    const int64_t dends[2] = {-512, 511}, lends[2] = {-32768, 32767};
    for (int de = 0; de < 2; ++de)
        for (int le = 0; le < 2; ++le) {
            for (int r = 0; r < 4; ++r) {
                digit[r].assign(kN, dends[de]);
                for (int o = 0; o < 4; ++o) limb[r][o].assign(kN, lends[le]);
            }
            char name[80];
            snprintf(name, sizeof name, "all digits %" PRId64 ", all limbs %" PRId64, dends[de], lends[le]);
            run(name, digit, limb);
        }
    // coherent sums: coefficient k0 of digit * limb is sum_{j <= k0} d[k0-j] l[j] - sum_{j > k0} d[k0-j+N] l[j];
    // with all digits -512 and limbs -32768 for j <= k0, +32767 for j > k0 every term has the same sign
    const int targets[5] = {0, 1, 511, 512, 1023};
    for (int t = 0; t < 5; ++t) {
        const int k0 = targets[t];
        for (int r = 0; r < 4; ++r) {
            digit[r].assign(kN, -512);
            for (int o = 0; o < 4; ++o)
                for (int j = 0; j < kN; ++j) limb[r][o][j] = j <= k0 ? -32768 : 32767;
        }
        char name[80];
        snprintf(name, sizeof name, "4,096 terms of coefficient %d aligned", k0);
        run(name, digit, limb);
    }
    // alternating extremes, rows and outputs out of phase with each other
    for (int r = 0; r < 4; ++r) {
        for (int j = 0; j < kN; ++j) digit[r][j] = ((j >> r) & 1) ? 511 : -512;
        for (int o = 0; o < 4; ++o)
            for (int j = 0; j < kN; ++j) limb[r][o][j] = (((j >> o) ^ r) & 1) ? 32767 : -32768;
    }
    run("alternating extremes", digit, limb);
    // random signs on extreme magnitudes
    for (int r = 0; r < 4; ++r) {
        for (int j = 0; j < kN; ++j) digit[r][j] = (next_u32() & 1) ? 511 : -512;
        for (int o = 0; o < 4; ++o)
            for (int j = 0; j < kN; ++j) limb[r][o][j] = (next_u32() & 1) ? 32767 : -32768;
    }
    run("extreme magnitudes, random signs", digit, limb);
    // a monomial digit: the product is a signed rotation of the limb polynomial
    for (int r = 0; r < 4; ++r) {
        digit[r].assign(kN, 0);
        digit[r][(301 * (r + 1)) % kN] = r & 1 ? -512 : 511;
    }
    run("monomial digits", digit, limb);

    printf("fft512 exactness: %s (largest distance from an integer %.3g)\n", wrong ? "FAILED" : "ok", worst);
    return wrong != 0 || !(worst < 1e-3);
}
