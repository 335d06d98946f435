// 512-point complex FFT held by one 64-lane wavefront, 8 points per lane, used to multiply
// polynomials of Z[X]/(X^1024+1) exactly.
//
// A real polynomial a of degree < N = 1024 is folded to z_j = (a_j + i a_{j+512}) psi^j,
// psi = exp(i pi / N) (the twist is applied inside pass 1); its 512-point DFT (kernel exp(+2 pi i jk/512)) holds the values of a
// at the roots psi^(4k+1) of X^N + 1 -- half of the roots, the others being the conjugates.
// Products of such values are the values of the product polynomial mod X^N + 1, and the
// inverse transform followed by the multiplication with psi^-j gives its coefficients back
// in the real and imaginary parts.
//
// The transform is radix 8 x 8 x 8.  Forward (decimation in frequency):
//   pass 1  lane L holds point L + 64 m, m = 0..7; twist, DFT over m, times w512^(L k0)
//   T1      through LDS: lane (k0, j0) receives the eight j1 values of row k0
//   pass 2  DFT over j1, times w64^(j0 k1)
//   T2      through LDS within groups of 8 lanes: lane (k0, k1) receives the eight j0 values
//   pass 3  DFT over j0: register k2 of lane (k0, k1) is frequency k0 + 8 k1 + 64 k2
// The inverse runs the same passes backwards with conjugate twiddles, so it consumes exactly
// the order the forward produces and no reordering is ever needed: spectra are stored and
// multiplied in "slot" order  slot = 64 * k2 + lane.
//
// Every function is a per-lane step; between a *_store and the matching *_load all lanes of
// the wave must have executed the store (the caller places the wave-level fence).  The same
// code compiles for the host, where a test drives the 64 lanes one after the other.
#pragma once
#include <hip/hip_runtime.h>

#ifndef FFT_HD
#define FFT_HD __host__ __device__ __forceinline__
#endif

namespace fft512 {

constexpr int kRowStride = 72;   // LDS row pitch in complex words: 64 + 8 keeps the 16-byte
constexpr int kGrpStride = 9;    // accesses of both transposes on distinct banks
constexpr int kBufWords = 8 * kRowStride;   // 576 complex words per wave

FFT_HD double2 cadd(double2 a, double2 b) { return make_double2(a.x + b.x, a.y + b.y); }
FFT_HD double2 csub(double2 a, double2 b) { return make_double2(a.x - b.x, a.y - b.y); }
FFT_HD double2 cmul(double2 a, double2 b) {
    return make_double2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
FFT_HD double2 cmulc(double2 a, double2 b) {   // a * conj(b)
    return make_double2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}

// y[k] = sum_m x[m] w^(m k), w = exp(+2 pi i / 8) (INV: exp(-2 pi i / 8)), in place.
template <bool INV>
FFT_HD void radix8(double2 (&x)[8]) {
    const double c = 0.70710678118654752440;
    double2 a0 = cadd(x[0], x[4]), a4 = csub(x[0], x[4]);
    double2 a1 = cadd(x[1], x[5]), a5 = csub(x[1], x[5]);
    double2 a2 = cadd(x[2], x[6]), a6 = csub(x[2], x[6]);
    double2 a3 = cadd(x[3], x[7]), a7 = csub(x[3], x[7]);
    // odd branch: a5 * w, a6 * w^2, a7 * w^3
    double2 b5, b6, b7;
    if (!INV) {
        b5 = make_double2((a5.x - a5.y) * c, (a5.x + a5.y) * c);
        b6 = make_double2(-a6.y, a6.x);
        b7 = make_double2((-a7.x - a7.y) * c, (a7.x - a7.y) * c);
    } else {
        b5 = make_double2((a5.x + a5.y) * c, (a5.y - a5.x) * c);
        b6 = make_double2(a6.y, -a6.x);
        b7 = make_double2((a7.y - a7.x) * c, (-a7.x - a7.y) * c);
    }
    // two 4-point DFTs with w4 = +-i
    {
        double2 c0 = cadd(a0, a2), c1 = csub(a0, a2), c2 = cadd(a1, a3), d = csub(a1, a3);
        double2 c3 = INV ? make_double2(d.y, -d.x) : make_double2(-d.y, d.x);
        x[0] = cadd(c0, c2); x[4] = csub(c0, c2); x[2] = cadd(c1, c3); x[6] = csub(c1, c3);
    }
    {
        double2 c0 = cadd(a4, b6), c1 = csub(a4, b6), c2 = cadd(b5, b7), d = csub(b5, b7);
        double2 c3 = INV ? make_double2(d.y, -d.x) : make_double2(-d.y, d.x);
        x[1] = cadd(c0, c2); x[5] = csub(c0, c2); x[3] = cadd(c1, c3); x[7] = csub(c1, c3);
    }
}

// psi^(64 m) = exp(i pi m / 16), m = 0..7: the part of the negacyclic twist psi^(L + 64 m) that
// does not depend on the lane.  It is applied to the inputs of pass 1; the lane's own psi^L is
// merged into the pass-1 twiddles.
FFT_HD double2 twist_const(int m) {
    const double c[8] = {1.0, 0.98078528040323044913, 0.92387953251128675613, 0.83146961230254523708,
                         0.70710678118654752440, 0.55557023301960222474, 0.38268343236508977173,
                         0.19509032201612826785};
    const double s[8] = {0.0, 0.19509032201612826785, 0.38268343236508977173, 0.55557023301960222474,
                         0.70710678118654752440, 0.83146961230254523708, 0.92387953251128675613,
                         0.98078528040323044913};
    return make_double2(c[m], s[m]);
}

// Per-lane constants, loaded once per kernel and kept in registers.
struct Lane {
    double2 tw1[8];    // psi^L * w512^(L k) = psi^(L (1 + 4k))
    double2 tw2[8];    // w64^((L & 7) k)    = psi^(32 (L & 7) k)
};

// tables[j] = psi^j = exp(i pi j / 1024), j < 2048
FFT_HD void lane_init(Lane &ln, const double2 *tables, int L) {
    for (int k = 0; k < 8; ++k) {
        ln.tw1[k] = tables[L * (1 + 4 * k)];
        ln.tw2[k] = tables[32 * (L & 7) * k];
    }
}

// ---- forward: x[m] holds the folded, untwisted point a[L + 64 m] + i a[L + 64 m + 512] -------
FFT_HD void fwd_pass1_store(double2 (&x)[8], const Lane &ln, double2 *buf, int L) {
    for (int m = 1; m < 8; ++m) x[m] = cmul(x[m], twist_const(m));
    radix8<false>(x);
    for (int k = 0; k < 8; ++k) buf[k * kRowStride + L] = cmul(x[k], ln.tw1[k]);
}
FFT_HD void fwd_pass2_load(double2 (&x)[8], const double2 *buf, int L) {
    const int row = (L >> 3) * kRowStride, j0 = L & 7;
    for (int j1 = 0; j1 < 8; ++j1) x[j1] = buf[row + j0 + 8 * j1];
    radix8<false>(x);
}
FFT_HD void fwd_pass2_store(const double2 (&x)[8], const Lane &ln, double2 *buf, int L) {
    const int row = (L >> 3) * kRowStride, j0 = L & 7;
    buf[row + j0] = x[0];
    for (int k = 1; k < 8; ++k) buf[row + k * kGrpStride + j0] = cmul(x[k], ln.tw2[k]);
}
FFT_HD void fwd_pass3(double2 (&x)[8], const double2 *buf, int L) {
    const int base = (L >> 3) * kRowStride + (L & 7) * kGrpStride;
    for (int j0 = 0; j0 < 8; ++j0) x[j0] = buf[base + j0];
    radix8<false>(x);
}

// ---- inverse (unnormalised: 512 times the folded, untwisted points come out) -----------
FFT_HD void inv_pass3_store(double2 (&x)[8], const Lane &ln, double2 *buf, int L) {
    radix8<true>(x);
    const int base = (L >> 3) * kRowStride + (L & 7) * kGrpStride;
    buf[base] = x[0];
    for (int j0 = 1; j0 < 8; ++j0) buf[base + j0] = cmulc(x[j0], ln.tw2[j0]);
}
FFT_HD void inv_pass2(double2 (&x)[8], const double2 *buf, int L) {
    const int row = (L >> 3) * kRowStride, j0 = L & 7;
    for (int k = 0; k < 8; ++k) x[k] = buf[row + k * kGrpStride + j0];
    radix8<true>(x);
}
FFT_HD void inv_pass2_store(const double2 (&x)[8], double2 *buf, int L) {
    const int row = (L >> 3) * kRowStride, j0 = L & 7;
    for (int j1 = 0; j1 < 8; ++j1) buf[row + j0 + 8 * j1] = x[j1];
}
FFT_HD void inv_pass1(double2 (&x)[8], const Lane &ln, const double2 *buf, int L) {
    for (int k = 0; k < 8; ++k) x[k] = cmulc(buf[k * kRowStride + L], ln.tw1[k]);
    radix8<true>(x);
    for (int m = 1; m < 8; ++m) x[m] = cmulc(x[m], twist_const(m));
}

}  // namespace fft512
