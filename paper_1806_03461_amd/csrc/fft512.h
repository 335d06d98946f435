// Four 512-point complex FFTs held by the four 64-lane wavefronts of a workgroup, 8 points per
// lane, used to multiply polynomials of Z[X]/(X^1024+1) exactly.
//
// A real polynomial a of degree < N = 1024 is folded to z_j = (a_j + i a_{j+512}) psi^j,
// psi = exp(i pi / N) (the twist is applied inside pass 1); its 512-point DFT (kernel
// exp(+2 pi i jk/512)) holds the values of a at the roots psi^(4k+1) of X^N + 1 -- half of the
// roots, the others being the conjugates.  Products of such values are the values of the product
// polynomial mod X^N + 1, and the inverse transform followed by the multiplication with psi^-j
// gives its coefficients back in the real and imaginary parts.
//
// The workgroup transforms four polynomials r = 0..3 at once and ends with every lane holding
// the spectra of all four at two frequencies, so that sums of products over r (the external
// product of a blind-rotation step) need no further exchange.  The transform is radix 8 x 8 x 8.
// Forward (decimation in frequency):
//   pass 1  wave r, lane L holds point L + 64 m of polynomial r, m = 0..7; twist, DFT over m
//           -> k0, times w512^(L k0); stored to row k0 of the polynomial's LDS buffer
//   ---- workgroup barrier ----
//           wave w takes rows k0 = 2w, 2w+1 of all four polynomials: lane (r, k0 & 1, j0) reads
//           the eight j1 values (L = j0 + 8 j1) of its row
//   pass 2  DFT over j1 -> k1, times w64^(j0 k1)
//   T2      through the lane's own row, inside groups of 8 lanes: lane (r, k0 & 1, k1) receives
//           the eight j0 values
//   pass 3  DFT over j0 -> k2: register k2 of that lane is frequency k0 + 8 k1 + 64 k2
//   gather  two register <-> lane-bit exchanges (lane bits 5 and 4, which hold r, against bits 2
//           and 1 of k2): register 2 r + q of lane (k2 >> 1, k0 & 1, k1) is polynomial r at
//           frequency k0 + 8 k1 + 64 k2, q = k2 & 1
// The inverse runs the same steps backwards with conjugate twiddles (scatter, pass 3, T2, pass 2
// into the rows, barrier, pass 1 by wave o for polynomial o), so it consumes exactly the order
// the forward produces and no reordering is ever needed.  Spectra are stored and multiplied in
// "slot" order: slot = 256 q + 64 w + lane.
//
// Rows 2w, 2w+1 of the four buffers are wave w's own between the two barriers (it is their only
// reader after the first and their only writer before the second), so T2 needs only wave-level
// fences.  Every function is a per-lane step; between a *_store and the matching load all lanes
// involved must have executed the store (the caller places the fence or barrier).  The same code
// compiles for the host, where a test drives the 256 lanes one after the other.
#pragma once
#include <hip/hip_runtime.h>

#ifndef FFT_HD
#define FFT_HD __host__ __device__ __forceinline__
#endif

namespace fft512 {

constexpr int kRowStride = 72;   // LDS row pitch in complex words: 64 + 8 keeps the 16-byte
constexpr int kGrpStride = 9;    // accesses of both transposes on distinct banks
// pitch between the four polynomials' buffers: 8 rows + 16 words, so that the lanes (r, k0 & 1, j0)
// of one access fall on 64 distinct 16-byte bank groups (592 = 16 mod 64)
constexpr int kPolyStride = 8 * kRowStride + 16;
constexpr int kBufWords = 4 * kPolyStride;   // complex words per workgroup

FFT_HD double2 cadd(double2 a, double2 b) { return make_double2(a.x + b.x, a.y + b.y); }
FFT_HD double2 csub(double2 a, double2 b) { return make_double2(a.x - b.x, a.y - b.y); }
FFT_HD double2 cmul(double2 a, double2 b) {
    return make_double2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
FFT_HD double2 cmulc(double2 a, double2 b) {   // a * conj(b)
    return make_double2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}

// y[k] = sum_m x[m] w^(m k), w = exp(+2 pi i / 8) (INV: exp(-2 pi i / 8)), in place.
// The odd branch needs a5 w and a7 w^3 with w = (1 + i) / sqrt 2: the factor 1 / sqrt 2 is not
// applied to them but folded into the fused multiply-adds of the last stage (16 operations for
// the four odd outputs instead of 20).
template <bool INV>
FFT_HD void radix8(double2 (&x)[8]) {
    const double c = 0.70710678118654752440;
    double2 a0 = cadd(x[0], x[4]), a4 = csub(x[0], x[4]);
    double2 a1 = cadd(x[1], x[5]), a5 = csub(x[1], x[5]);
    double2 a2 = cadd(x[2], x[6]), a6 = csub(x[2], x[6]);
    double2 a3 = cadd(x[3], x[7]), a7 = csub(x[3], x[7]);
    // even outputs: a 4-point DFT with w4 = +-i
    {
        double2 c0 = cadd(a0, a2), c1 = csub(a0, a2), c2 = cadd(a1, a3), d = csub(a1, a3);
        double2 c3 = INV ? make_double2(d.y, -d.x) : make_double2(-d.y, d.x);
        x[0] = cadd(c0, c2); x[4] = csub(c0, c2); x[2] = cadd(c1, c3); x[6] = csub(c1, c3);
    }
    // odd outputs: s5 = sqrt 2 * a5 w, b6 = a6 w^2, s7 = sqrt 2 * a7 w^3 (conjugate w for INV)
    double2 s5, b6, s7;
    if (!INV) {
        s5 = make_double2(a5.x - a5.y, a5.x + a5.y);
        b6 = make_double2(-a6.y, a6.x);
        s7 = make_double2(-a7.x - a7.y, a7.x - a7.y);
    } else {
        s5 = make_double2(a5.x + a5.y, a5.y - a5.x);
        b6 = make_double2(a6.y, -a6.x);
        s7 = make_double2(a7.y - a7.x, -a7.x - a7.y);
    }
    {
        const double2 c0 = cadd(a4, b6), c1 = csub(a4, b6), t = cadd(s5, s7), u = csub(s5, s7);
        // x1, x5 = c0 +- c t;  x3, x7 = c1 +- c (+-i u)
        x[1] = make_double2(fma(c, t.x, c0.x), fma(c, t.y, c0.y));
        x[5] = make_double2(fma(-c, t.x, c0.x), fma(-c, t.y, c0.y));
        if (!INV) {
            x[3] = make_double2(fma(-c, u.y, c1.x), fma(c, u.x, c1.y));
            x[7] = make_double2(fma(c, u.y, c1.x), fma(-c, u.x, c1.y));
        } else {
            x[3] = make_double2(fma(c, u.y, c1.x), fma(-c, u.x, c1.y));
            x[7] = make_double2(fma(-c, u.y, c1.x), fma(c, u.x, c1.y));
        }
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

// The row lane L of wave w works in between the two barriers: row 2w + (L >> 3 & 1) of
// polynomial L >> 4, as an offset in complex words from the start of the four buffers.
FFT_HD int row_of(int w, int L) { return (L >> 4) * kPolyStride + (2 * w + ((L >> 3) & 1)) * kRowStride; }

// ---- forward: x[m] holds the folded, untwisted point a[L + 64 m] + i a[L + 64 m + 512] -------
// wave r, into its polynomial's buffer
FFT_HD void fwd_pass1_store(double2 (&x)[8], const Lane &ln, double2 *poly, int L) {
    for (int m = 1; m < 8; ++m) x[m] = cmul(x[m], twist_const(m));
    radix8<false>(x);
    for (int k = 0; k < 8; ++k) poly[k * kRowStride + L] = cmul(x[k], ln.tw1[k]);
}
// wave w, on its rows (row = buffers + row_of(w, L))
FFT_HD void fwd_pass2_load(double2 (&x)[8], const double2 *row, int L) {
    const int j0 = L & 7;
    for (int j1 = 0; j1 < 8; ++j1) x[j1] = row[j0 + 8 * j1];
    radix8<false>(x);
}
FFT_HD void fwd_pass2_store(const double2 (&x)[8], const Lane &ln, double2 *row, int L) {
    const int j0 = L & 7;
    row[j0] = x[0];
    for (int k = 1; k < 8; ++k) row[k * kGrpStride + j0] = cmul(x[k], ln.tw2[k]);
}
FFT_HD void fwd_pass3(double2 (&x)[8], const double2 *row, int L) {
    const int base = (L & 7) * kGrpStride;
    for (int j0 = 0; j0 < 8; ++j0) x[j0] = row[base + j0];
    radix8<false>(x);
}

// ---- inverse (unnormalised: 512 times the folded, untwisted points come out) -----------
FFT_HD void inv_pass3_store(double2 (&x)[8], const Lane &ln, double2 *row, int L) {
    radix8<true>(x);
    const int base = (L & 7) * kGrpStride;
    row[base] = x[0];
    for (int j0 = 1; j0 < 8; ++j0) row[base + j0] = cmulc(x[j0], ln.tw2[j0]);
}
FFT_HD void inv_pass2(double2 (&x)[8], const double2 *row, int L) {
    const int j0 = L & 7;
    for (int k = 0; k < 8; ++k) x[k] = row[k * kGrpStride + j0];
    radix8<true>(x);
}
FFT_HD void inv_pass2_store(const double2 (&x)[8], double2 *row, int L) {
    const int j0 = L & 7;
    for (int j1 = 0; j1 < 8; ++j1) row[j0 + 8 * j1] = x[j1];
}
// wave o, from its polynomial's buffer
FFT_HD void inv_pass1(double2 (&x)[8], const Lane &ln, const double2 *poly, int L) {
    for (int k = 0; k < 8; ++k) x[k] = cmulc(poly[k * kRowStride + L], ln.tw1[k]);
    radix8<true>(x);
    for (int m = 1; m < 8; ++m) x[m] = cmulc(x[m], twist_const(m));
}

// ---- gather / scatter: registers <-> lane bits 5 and 4 -----------------------------------
// One exchange step on a pair of 32-bit registers (a, b) of all lanes, lane bit `bit` (5 or 4):
// afterwards a holds, in lanes with the bit clear, what it held, and in lanes with the bit set,
// what b held in the partner lane (bit clear); b holds, in lanes with the bit clear, what a held
// in the partner lane (bit set), and in lanes with the bit set, what it held.  Applying the step
// twice restores both registers.  On the device this is one v_permlane32_swap / v_permlane16_swap.
#if defined(__HIPCC__)
template <int BIT>
__device__ __forceinline__ void lane_bit_swap(uint32_t &a, uint32_t &b) {
    static_assert(BIT == 5 || BIT == 4, "lane bit 5 or 4");
#if defined(__HIP_DEVICE_COMPILE__)
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    u32x2 r;
    if (BIT == 5) r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    else r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
    a = r[0]; b = r[1];
#else
    (void)a; (void)b;      // the host pass only parses device code
#endif
}
template <int BIT>
__device__ __forceinline__ void lane_bit_swap(double2 &a, double2 &b) {
    uint32_t wa[4] = {(uint32_t)__double2loint(a.x), (uint32_t)__double2hiint(a.x),
                      (uint32_t)__double2loint(a.y), (uint32_t)__double2hiint(a.y)};
    uint32_t wb[4] = {(uint32_t)__double2loint(b.x), (uint32_t)__double2hiint(b.x),
                      (uint32_t)__double2loint(b.y), (uint32_t)__double2hiint(b.y)};
    for (int q = 0; q < 4; ++q) lane_bit_swap<BIT>(wa[q], wb[q]);
    a = make_double2(__hiloint2double((int)wa[1], (int)wa[0]), __hiloint2double((int)wa[3], (int)wa[2]));
    b = make_double2(__hiloint2double((int)wb[1], (int)wb[0]), __hiloint2double((int)wb[3], (int)wb[2]));
}
// In: register k2 of lane (r, k0 & 1, k1).  Out: register 2 r + (k2 & 1) of lane (k2 >> 1, k0 & 1, k1).
__device__ __forceinline__ void gather_rows(double2 (&x)[8]) {
    for (int k = 0; k < 4; ++k) lane_bit_swap<5>(x[k], x[k + 4]);
    for (int k = 0; k < 2; ++k) { lane_bit_swap<4>(x[k], x[k + 2]); lane_bit_swap<4>(x[k + 4], x[k + 6]); }
}
// the inverse of gather_rows (the same exchanges in reverse order)
__device__ __forceinline__ void scatter_rows(double2 (&x)[8]) {
    for (int k = 0; k < 2; ++k) { lane_bit_swap<4>(x[k], x[k + 2]); lane_bit_swap<4>(x[k + 4], x[k + 6]); }
    for (int k = 0; k < 4; ++k) lane_bit_swap<5>(x[k], x[k + 4]);
}
#endif

// The same exchanges written out over the registers of a whole wave (x[lane][register]), for
// host code that drives the lanes one after the other.
inline void gather_rows_wave(double2 (*x)[8]) {
    for (int bit = 5; bit >= 4; --bit) {
        const int d = 1 << bit, rs = bit == 5 ? 4 : 2;      // lane distance, register distance
        for (int L = 0; L < 64; ++L) {
            if (L & d) continue;
            for (int k = 0; k < 8; ++k) {
                if (k & rs) continue;
                const double2 t = x[L][k + rs];
                x[L][k + rs] = x[L + d][k];
                x[L + d][k] = t;
            }
        }
    }
}
inline void scatter_rows_wave(double2 (*x)[8]) {
    for (int bit = 4; bit <= 5; ++bit) {
        const int d = 1 << bit, rs = bit == 5 ? 4 : 2;
        for (int L = 0; L < 64; ++L) {
            if (L & d) continue;
            for (int k = 0; k < 8; ++k) {
                if (k & rs) continue;
                const double2 t = x[L][k + rs];
                x[L][k + rs] = x[L + d][k];
                x[L + d][k] = t;
            }
        }
    }
}

}  // namespace fft512
