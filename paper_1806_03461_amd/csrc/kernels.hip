// gfx950 kernels: transform-domain bootstrapping key, blind rotation, key switch, output gather.
//
// The bootstrapped gate is the CGGI gate the TAPAS paper builds its circuits from
// (Sec. 3.1.2, Sec. 4.1); the paper gives no construction, the steps are the public ones.
//
// Exactness.  Each blind-rotation step needs, for both TRLWE components c,
//     sum_{r<4} digit_r(X) * BK_i[r][c](X)   mod (X^1024 + 1, 2^32),
// digit_r with coefficients in [-512, 512).  Every 32-bit key coefficient is split into two
// signed 16-bit limbs, key = lo + 2^16 hi (mod 2^32); the two integer products
// sum_r digit_r * lo_r and sum_r digit_r * hi_r have coefficients below 2^36 in magnitude and
// are computed with double-precision FFTs whose rounding error stays orders of magnitude below
// 1/2, so rounding the inverse transform to the nearest integer gives them exactly; the result
// is lo-sum + 2^16 * hi-sum (mod 2^32).  MI355X issues FP64 FMAs at full vector rate, which
// makes this cheaper than any 32-bit-integer number-theoretic transform on its VALU.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstddef>
#include <cstdlib>

#include "common.h"
#include "fft512.h"
#include "kernels.h"

namespace tfhe {

using namespace fft512;

namespace {

constexpr int kN = 1024;
constexpr int kHalf = 512;
constexpr int kThreadsPerGate = 256;
constexpr uint32_t kEighth = 1u << 29;

__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ------------------------------------------------------------------------------------------
// Bootstrapping key -> transform domain.  One workgroup per sample row (i, r): its four waves
// transform the four polynomials o = 2*component + limb with the very steps the blind rotation
// applies to its four digit polynomials, so the spectra land in the slot order the products use.
// bk_raw [n][4][2][1024] uint32  ->  bk_fft [n][4][o][512] complex.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bk_to_spectrum_kernel(const uint32_t *__restrict__ bk_raw,
                                                             double2 *__restrict__ bk_fft,
                                                             const double2 *__restrict__ tables) {
    __shared__ double2 buf[kBufWords];
    const int L = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const size_t row = blockIdx.x;                 // i * 4 + r
    const int c = wv >> 1, limb = wv & 1;          // pass 1: wave o = 2 c + limb
    const uint32_t *src = bk_raw + (row * 2 + (size_t)c) * kN;
    Lane ln;
    lane_init(ln, tables, L);
    double2 x[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) {
        const int j = L + 64 * m;
        int32_t v[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t w = src[j + h * kHalf];
            const int32_t lo = (int16_t)(w & 0xFFFFu);
            const int32_t hi = (int16_t)(((w - (uint32_t)lo) >> 16) & 0xFFFFu);
            v[h] = limb ? hi : lo;
        }
        // the 1/512 of the inverse transform is folded into the key (exact: a power of two)
        x[m] = make_double2((double)v[0] * (1.0 / 512.0), (double)v[1] * (1.0 / 512.0));
    }
    fwd_pass1_store(x, ln, buf + wv * kPolyStride, L);
    __syncthreads();
    double2 *mine = buf + row_of(wv, L);
    fwd_pass2_load(x, mine, L);
    wave_sync();
    fwd_pass2_store(x, ln, mine, L);
    wave_sync();
    fwd_pass3(x, mine, L);
    gather_rows(x);
#pragma unroll
    for (int o = 0; o < 4; ++o)
#pragma unroll
        for (int q = 0; q < 2; ++q)
            bk_fft[(row * 4 + (size_t)o) * kHalf + 256 * q + threadIdx.x] = x[2 * o + q];
}

// ------------------------------------------------------------------------------------------
// Blind rotation, one gate per workgroup of 256 threads (4 waves).
//   prologue  c = (0, kappa) + m (s0 c0 + s1 c1); abar_j = round(c_j * 2N / 2^32); ACC = (0, X^-bbar v)
//   n steps   D = X^abar_i ACC - ACC; wave r = (component, digit) decomposes its digit polynomial
//             and runs pass 1 of its forward FFT; after a barrier wave w carries the frequencies
//             k0 = 2w, 2w+1 of all four polynomials through passes 2 and 3, gathers the four
//             spectra of each of its frequencies into one lane, multiplies them with the key row
//             in registers, scatters the four output spectra o = (component, limb) back and runs
//             the inverse passes 3 and 2; after a second barrier wave o runs inverse pass 1,
//             rounds and adds into ACC; a third barrier closes the step
//   epilogue  sample extraction of coefficient 0 -> ext[gate][1025]
// A workgroup takes gates blockIdx.x, blockIdx.x + gridDim.x, ...; launches normally have one
// workgroup per gate (see resident_groups()).
// ------------------------------------------------------------------------------------------
constexpr int kMirror = 64;       // coefficients 0..63 of each accumulator component are kept a second time
struct GateLds {
    // accumulator (mask, body), stored bitwise complemented: c = ~ACC = -ACC - 1.  Behind each component
    // sits a mirror of its first 64 coefficients, stored as -c - 2: a rotated read of 64 consecutive
    // coefficients that runs past X^N continues into the mirror, and the value found there already
    // carries the sign change of X^N = -1 (see the rotation in blind_rotate_body)
    uint32_t acc[2][kN + kMirror];
    double2 buf[kBufWords];       // the four polynomials' transform buffers
    uint16_t bar[1032];           // abar_0 .. abar_{n-1}, bbar
};

__device__ __forceinline__ void gate_constants(int op, uint32_t &kappa, uint32_t &mult) {
    switch (op) {
    case TFHE_NAND: kappa = kEighth;          mult = 0xFFFFFFFFu; break;
    case TFHE_AND:  kappa = 0u - kEighth;     mult = 1u;          break;
    case TFHE_OR:   kappa = kEighth;          mult = 1u;          break;
    case TFHE_NOR:  kappa = 0u - kEighth;     mult = 0xFFFFFFFFu; break;
    case TFHE_XOR:  kappa = 2u * kEighth;     mult = 2u;          break;
    default:        kappa = 0u - 2u * kEighth; mult = 0xFFFFFFFEu; break;   // XNOR
    }
}

// 16-byte load from a buffer: descriptor and soffset are scalar, voffset is the lane's byte offset
__device__ __forceinline__ double2 load_key(__amdgpu_buffer_rsrc_t rsrc, uint32_t voffset, uint32_t soffset) {
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voffset, (int)soffset, 0);
    double2 out;
    out.x = __hiloint2double((int)v.y, (int)v.x);
    out.y = __hiloint2double((int)v.w, (int)v.z);
    return out;
}

// A step's key values of one thread come in four parts of 8 (32 registers): part p = 2 q + h holds
// rows r = 0..3 x outputs o = 2h, 2h+1 at the thread's slot 256 q + tid.
// AHEAD: the latency variant (launches that leave one workgroup per CU) requests the whole key
// row of step i + 1 while step i still runs, in eight portions of four loads placed between the
// phases that follow the products of step i: a portion keeps the CU's one address unit busy for
// 4 x 16 clocks per wave, and a wave alone on its SIMD cannot issue anything else meanwhile, so
// portions issued back to back stall all four waves (measured on 64 gates: all 32 loads in one
// place 2.06 ms, two places 1.82 ms, four 1.71 ms, eight 1.62 ms; no key traffic at all 1.50 ms).
// At full occupancy other workgroups cover the loads and holding registers for them does not pay:
// with two parts kept in flight (registers freed by moving the pass-2 twiddles to LDS) a launch of
// 65,536 gates took 390-410 ms instead of 266-278.  The wait for a key row that no workgroup of the
// XCD has touched yet is what keeps the workgroups of an XCD within the few rows its L2 holds.
template <bool MARGIN, int AHEAD>
__device__ __forceinline__ void blind_rotate_body(const BlindRotateArgs &a) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    GateLds &my = *reinterpret_cast<GateLds *>(lds_raw);
    static_assert(AHEAD == 0 || AHEAD == 4, "no key values or a whole step's ahead");

    const int tid = threadIdx.x;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave, in a scalar register
    const int L = tid & 63;

    Lane ln;
    lane_init(ln, a.tables, L);
    const __amdgpu_buffer_rsrc_t key_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<double2 *>(a.bk_fft), 0, (int)((size_t)a.n * 16 * kHalf * sizeof(double2)), 0x00020000);
    const uint32_t voff = (uint32_t)tid * (uint32_t)sizeof(double2);
    auto key_offset = [](int row, int part, int r, int o2) {
        return (uint32_t)row * 16u * kHalf * (uint32_t)sizeof(double2) +
               (uint32_t)(((r * 4 + 2 * (part & 1) + o2) * kHalf + 256 * (part >> 1)) * sizeof(double2));
    };

    const int comp = wv >> 1;                   // pass 1 forward: component of D; inverse: component of ACC
    const int sel = wv & 1;                     // pass 1 forward: digit index; inverse: limb
    // Signed digit `sel` of x: add the rounding constant and the half-bases of the lower digits
    // (not its own: its two's-complement field then already is the centred digit), move the
    // field to the top of the word, shift back down arithmetically.
    const uint32_t dround = 1u << (31 - 2 * a.bgbit);
    const uint32_t doffset = sel ? dround : dround + (1u << (31 - a.bgbit));
    const uint32_t dfield = (uint32_t)(32 - a.bgbit * (1 + sel));   // lowest bit of the digit's field
    double2 *const poly = my.buf + wv * kPolyStride;      // pass 1: this wave's polynomial
    double2 *const mine = my.buf + row_of(wv, L);         // passes 2, 3: this lane's row
    double worst = 0.0;
    // Wave priority, throughput kernel only (three workgroups share a CU): the phases that lead up to
    // a barrier or follow one directly -- rotation and forward pass 1, forward passes 2 and 3, inverse
    // pass 1 and the accumulation -- issue ahead of the other workgroups' gather, products and
    // scatter, which wait on swaps and key loads anyway.  Measured: 3-4 % (12,288 gates 55.0 -> 53.3 ms,
    // 65,536 gates 286 -> 276 ms); raising the priority at the gather instead costs up to 30 %.
    auto priority = [](int level) {
        if (AHEAD) return;               // a lone workgroup per CU has nobody to overtake
        if (level) __builtin_amdgcn_s_setprio(2);
        else __builtin_amdgcn_s_setprio(0);
    };

    for (size_t gi = blockIdx.x; gi < a.count; gi += gridDim.x) {
    // ---- prologue ----
    {
        int op = a.uniform_op;
        size_t i0 = gi, i1 = gi;
        uint32_t s0 = 1u, s1 = 1u;
        const uint32_t *src1 = a.in1;
        if (a.recs) {
            const tfhe_gate_rec r = a.recs[gi];
            op = r.op; i0 = (size_t)r.in0; i1 = (size_t)r.in1;
            s0 = r.neg0 ? 0xFFFFFFFFu : 1u; s1 = r.neg1 ? 0xFFFFFFFFu : 1u;
        } else if (op == TFHE_MUX) {
            i0 = i1 = gi >> 1;
            if (gi & 1) { op = TFHE_MUX_ELSE; src1 = a.in1_alt; }
        }
        // a multiplexer half is an AND whose result stays under the ring key:
        // AND(s, a), then AND(NOT s, b)
        if (op == TFHE_MUX_ELSE) s0 = 0u - s0;
        if (op >= TFHE_MUX) op = TFHE_AND;
        uint32_t kappa, mult;
        gate_constants(op, kappa, mult);
        const size_t w = (size_t)a.n + 1;
        for (int j = tid; j <= a.n; j += kThreadsPerGate) {
            uint32_t c = mult * (s0 * a.in0[i0 * w + j] + s1 * src1[i1 * w + j]);
            if (j == a.n) c += kappa;
            my.bar[j] = (uint16_t)(((c + (1u << 20)) >> 21) & 2047u);
        }
    }
    __syncthreads();
    {
        const int bbar = my.bar[a.n];
        const int bb = bbar & (kN - 1);
        const uint32_t first = bbar < kN ? kEighth : 0u - kEighth;   // X^-bbar v, closed form
        for (int j = tid; j < kN; j += kThreadsPerGate) {
            const uint32_t c = ~(j < kN - bb ? first : 0u - first);
            my.acc[0][j] = ~0u;
            my.acc[1][j] = c;
            if (j < kMirror) { my.acc[0][kN + j] = 0u - ~0u - 2u; my.acc[1][kN + j] = 0u - c - 2u; }
        }
    }
    __syncthreads();

    double2 ahead[AHEAD ? AHEAD : 1][4][2];     // [part][row][output of the pair]
    // portion e of 8: rows 2 (e & 1), 2 (e & 1) + 1 of part e >> 1
    auto load_ahead = [&](int row, int e) {
        if (!AHEAD) return;
#pragma unroll
        for (int r = 2 * (e & 1); r < 2 * (e & 1) + 2; ++r)
#pragma unroll
            for (int o2 = 0; o2 < 2; ++o2)
                ahead[e >> 1][r][o2] = load_key(key_rsrc, voff, key_offset(row, e >> 1, r, o2));
    };
#pragma unroll
    for (int e = 0; e < 8; ++e) load_ahead(0, e);

    int abar_next = my.bar[0];
    for (int i = 0; i < a.n; ++i) {
        double2 x[8];
        priority(1);
        {
        // ---- rotate, subtract, decompose, fold and twist ----
        // read one step ahead (off the critical path); the same in every lane, so it goes to a scalar
        // register and everything below that does not depend on the lane is scalar arithmetic
        const int abar = __builtin_amdgcn_readfirstlane(abar_next);
        typedef __attribute__((address_space(3))) const uint32_t lds_word;
        const uint32_t acc_at = (uint32_t)(uintptr_t)(lds_word *)my.acc[comp];
        const uint32_t lane4 = (uint32_t)L << 2;
        const uint32_t back4 = (uint32_t)(0 - abar) << 2;       // X^abar reads abar coefficients back, mod 8192 bytes
        // Coefficient j = L + 64 m + 512 h of X^abar ACC is +-ACC[(j - abar) mod N].  The 64 lanes read 64
        // consecutive source coefficients starting at lane 0's, whose byte offset and sign are scalar.  The
        // run wraps past X^N in exactly one of the sixteen (m, h), from some lane on; those lanes read
        // on into the mirror behind the component, which holds mu = -c - 2 for the first 64 coefficients.
        // With ACC stored as c = ~ACC, the step's  +-ACC[src] - ACC[j] + doffset  is
        //   source not past X^N (flip = ~0):  -c[src] + c[j] + doffset = (c[src] ^ ~0) + c[j] + doffset + 1
        //   source past X^N (flip = 0):        c[src] + c[j] + doffset + 2
        // i.e. (c[src] ^ flip) + c[j] + (doffset + 2 + flip); a lane in the mirror needs the other flip,
        // and (mu ^ flip) + flip = (c ^ ~flip) + ~flip for either flip: two vector instructions per
        // coefficient, whatever the lane.
        uint32_t from[8][2], flip[8][2], bias[8][2];
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                // + 4096: bit 12 of the sum then says "lane 0's source not past X^N"
                const uint32_t s = back4 + (uint32_t)(64 * m + h * kHalf) * 4u + 4096u;
                from[m][h] = acc_at + (s & 4095u);
                flip[m][h] = (uint32_t)((int32_t)(s << 19) >> 31);
                bias[m][h] = doffset + 2u + flip[m][h];
                asm("" : "+s"(from[m][h]), "+s"(flip[m][h]), "+s"(bias[m][h]));
            }
        // all sixteen rotated reads are issued before any of them is consumed
        uint32_t rot[8][2];
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                rot[m][h] = *(lds_word *)(uintptr_t)(lane4 + from[m][h]);
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            int32_t dig[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int j = L + 64 * m + h * kHalf;
                const uint32_t d = (rot[m][h] ^ flip[m][h]) + my.acc[comp][j] + bias[m][h];
                dig[h] = __builtin_amdgcn_sbfe((int32_t)d, dfield, (uint32_t)a.bgbit);    // signed field
            }
            x[m] = make_double2((double)dig[0], (double)dig[1]);
        }
        }
        if (i > 0) load_ahead(i, 6);
        fwd_pass1_store(x, ln, poly, L);
        __syncthreads();
        if (i > 0) load_ahead(i, 7);

        // ---- this wave's frequencies of all four polynomials ----
        fwd_pass2_load(x, mine, L);
        wave_sync();
        fwd_pass2_store(x, ln, mine, L);
        wave_sync();
        fwd_pass3(x, mine, L);
        priority(0);
        gather_rows(x);                      // x[2 r + q]: digit polynomial r at slot 256 q + tid

        // ---- products with the key row, in registers: y[2 o + q] = sum_r x[2 r + q] key[r][o] ----
        double2 y[8];
#pragma unroll
        for (int part = 0; part < 4; ++part) {
            const int q = part >> 1;
            double2 k[4][2];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int o2 = 0; o2 < 2; ++o2)
                    k[r][o2] = part < AHEAD ? ahead[part < AHEAD ? part : 0][r][o2]
                                            : load_key(key_rsrc, voff, key_offset(i, part, r, o2));
#pragma unroll
            for (int o2 = 0; o2 < 2; ++o2) {
                // one chain of fused multiply-adds per real output (four independent chains per part)
                const double2 d0 = x[q];
                double yr = d0.x * k[0][o2].x, yi = d0.x * k[0][o2].y;
                yr = fma(-d0.y, k[0][o2].y, yr);
                yi = fma(d0.y, k[0][o2].x, yi);
#pragma unroll
                for (int r = 1; r < 4; ++r) {
                    const double2 d = x[2 * r + q];
                    yr = fma(d.x, k[r][o2].x, yr);
                    yi = fma(d.x, k[r][o2].y, yi);
                    yr = fma(-d.y, k[r][o2].y, yr);
                    yi = fma(d.y, k[r][o2].x, yi);
                }
                y[2 * (2 * (part & 1) + o2) + q] = make_double2(yr, yi);
            }
        }
        const int next = i + 1 < a.n ? i + 1 : i;     // the last step requests its own row again
        load_ahead(next, 0);

        // ---- back: scatter the four output spectra to their lanes, inverse passes 3 and 2 ----
        scatter_rows(y);
        inv_pass3_store(y, ln, mine, L);
        wave_sync();
        load_ahead(next, 1);
        inv_pass2(y, mine, L);
        wave_sync();
        load_ahead(next, 2);
        inv_pass2_store(y, mine, L);
        __syncthreads();
        abar_next = my.bar[i + 1];           // bar[n] exists (it holds bbar)
        load_ahead(next, 3);

        // ---- inverse pass 1 of output polynomial o = wave, exact rounding, accumulate ----
        priority(1);
        inv_pass1(x, ln, poly, L);
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            const double part[2] = {x[m].x, x[m].y};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                // 1.5 * 2^52 - part leaves round-to-nearest(-part) = -round(part) mod 2^32 in the low word
                // (ties go to even either way); the complemented accumulator takes it: ~(ACC + r) = ~ACC - r
                const double shifted = 6755399441055744.0 - part[h];
                uint32_t r = (uint32_t)__double2loint(shifted);
                if (MARGIN) worst = fmax(worst, fabs(part[h] + (shifted - 6755399441055744.0)));
                if (sel) r <<= 16;
                if (m == 3 && h == 1) load_ahead(next, 4);
                atomicAdd(&my.acc[comp][L + 64 * m + h * kHalf], r);
                if (m == 0 && h == 0) atomicSub(&my.acc[comp][kN + L], r);      // the mirror holds -c - 2
            }
        }
        __syncthreads();
        load_ahead(next, 5);
    }

    // ---- epilogue: the constant coefficient as an LWE sample under the ring key ----
    {
        uint32_t *ext = a.ext + gi * (size_t)(kN + 1);
        // ACC = ~c, -ACC = c + 1
        for (int j = tid; j < kN; j += kThreadsPerGate) ext[j] = j == 0 ? ~my.acc[0][0] : my.acc[0][kN - j] + 1u;
        if (tid == 0) ext[kN] = ~my.acc[1][0];
    }
    __syncthreads();          // the next gate's prologue overwrites the accumulator
    }
    if (MARGIN) {
        // non-negative doubles order like their bit patterns
        atomicMax(reinterpret_cast<unsigned long long *>(a.margin),
                  (unsigned long long)__double_as_longlong(worst));
    }
}

template <bool MARGIN>
__global__ __launch_bounds__(kThreadsPerGate) __attribute__((amdgpu_waves_per_eu(3, 3))) void blind_rotate_kernel(BlindRotateArgs a) {
    blind_rotate_body<MARGIN, 0>(a);
}

// The same step for batches of at most one gate per CU, where a gate's latency is all that
// counts: the whole key row of step i + 1 is requested while step i still runs.
template <bool MARGIN>
__global__ __launch_bounds__(kThreadsPerGate) __attribute__((amdgpu_waves_per_eu(1, 1))) void blind_rotate_latency_kernel(BlindRotateArgs a) {
    blind_rotate_body<MARGIN, 4>(a);
}

// ------------------------------------------------------------------------------------------
// Key switch, one workgroup per gate:  out = (0, b') - sum_{i,j} KSK[i][j][digit_ij]
// over the t base-2^basebit digits of the rounded mask words; digit 0 reads the zero row
// appended to the key so that all loads of one mask word can be in flight together.
// ------------------------------------------------------------------------------------------
template <int T>
__global__ __launch_bounds__(256) void key_switch_kernel(KeySwitchArgs a) {
    __shared__ uint32_t ext[kN + 1];
    const int tid = threadIdx.x;
    // with a.splits > 1 the mask words of one gate are shared out over that many workgroups,
    // each adding its partial result into the (zeroed) output with integer atomics
    const size_t gi = blockIdx.x / a.splits;
    const int part = (int)(blockIdx.x % a.splits);
    // the second half of a multiplexer has been added into the first: nothing to switch
    if (a.recs ? a.recs[gi].op == TFHE_MUX_ELSE : (a.uniform_mux && (gi & 1))) return;
    const uint32_t *src = a.ext + gi * (size_t)(kN + 1);
    for (int j = tid; j <= kN; j += 256) ext[j] = src[j];
    __syncthreads();

    const int words = a.n + 1;
    constexpr int kMaxPerThread = 5;              // ceil(1025 / 256)
    uint32_t acc[kMaxPerThread];
#pragma unroll
    for (int q = 0; q < kMaxPerThread; ++q) {
        const int w = tid + 256 * q;
        acc[q] = (w == a.n && part == 0) ? ext[kN] : 0u;
    }
    const int values = (1 << a.basebit) - 1;
    const uint32_t round = 1u << (31 - T * a.basebit);
    const size_t zero_row = (size_t)kN * T * values;   // appended row of zeros
    const int per_thread = (words + 255) >> 8;
    const int i_begin = part * (kN / a.splits), i_end = i_begin + kN / a.splits;
    for (int i = i_begin; i < i_end; ++i) {
        const uint32_t ai = ext[i] + round;
        const uint32_t *rows[T];
#pragma unroll
        for (int j = 0; j < T; ++j) {
            const uint32_t v = (ai >> (32 - a.basebit * (j + 1))) & (uint32_t)values;
            const size_t row = v ? ((size_t)i * T + j) * values + (v - 1) : zero_row;
            rows[j] = a.ksk + row * (size_t)a.stride;
        }
        for (int q = 0; q < per_thread; ++q) {
            const int w = tid + 256 * q;
            if (w < words) {
                uint32_t part_sum[T];
#pragma unroll
                for (int j = 0; j < T; ++j) part_sum[j] = rows[j][w];
                uint32_t sum = 0;
#pragma unroll
                for (int j = 0; j < T; ++j) sum += part_sum[j];
                acc[q] -= sum;
            }
        }
    }
    const size_t out_index = a.recs ? (size_t)a.recs[gi].out : (a.uniform_mux ? gi >> 1 : gi);
    uint32_t *out = a.out + out_index * (size_t)words;
#pragma unroll
    for (int q = 0; q < kMaxPerThread; ++q) {
        const int w = tid + 256 * q;
        if (w < words) {
            if (a.splits > 1) atomicAdd(out + w, acc[q]);
            else out[w] = acc[q];
        }
    }
}

// zero the output samples that the split key switch accumulates into
__global__ void zero_outputs_kernel(KeySwitchArgs a) {
    const size_t gi = blockIdx.x;
    if (a.recs ? a.recs[gi].op == TFHE_MUX_ELSE : (a.uniform_mux && (gi & 1))) return;
    const size_t out_index = a.recs ? (size_t)a.recs[gi].out : (a.uniform_mux ? gi >> 1 : gi);
    uint32_t *out = a.out + out_index * (size_t)(a.n + 1);
    for (int w = threadIdx.x; w <= a.n; w += blockDim.x) out[w] = 0u;
}

// ------------------------------------------------------------------------------------------
// Key switch of large batches as a dense contraction on the matrix cores (t = 8 digits in base
// 4, N = 1024, n + 1 <= 512).  With one-hot digits the sum is a matrix product
//     S[g][c] = sum_{i, j, v} [digit_ij(g) == v] * KSK[i][j][v][c]      (v = 0: a zero row)
// with K = 1024 * 8 * 4 = 32,768.  The 32-bit key words are split into four balanced signed
// bytes, x = s0 + 2^8 s1 + 2^16 s2 + 2^24 s3 (mod 2^32), |s| <= 128, so every plane is an exact
// int8 x int8 -> int32 product (|sum| <= 2^20) and S is recombined with shifts.
//
// v_mfma_i32_32x32x32_i8: lane l supplies row (A) / column (B) l % 32 and the 16 bytes of
// k-group l / 32; both operands use the same byte <-> k map, which is all the contraction needs.
// One k-step of 32 is one mask word i: its 8 digits x 4 values.  A lane's A operand is built
// in registers: 4 digits -> 4 words 1 << (8 * digit).  The key is pre-tiled so that a B operand
// (32 columns x 32 k) is 1 KB contiguous in lane order: tiles[block of 32 words][i][plane][lane].
//
// Workgroup = 4 waves = 256 gates x 64 output words; wave = 128 gates x 32 words x 4 planes =
// 16 accumulator tiles (256 registers): per mask word 4 B tiles are loaded and 16 MFMAs issued.
// ------------------------------------------------------------------------------------------
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kKsRows = 256;      // gates per workgroup
constexpr int kKsChunk = 128;     // mask words staged per round (132 KB of LDS: one workgroup per CU anyway)
constexpr int kKsAhead = 8;       // mask words whose key tiles are in flight

struct KsMatrixLds {
    uint32_t mask_words[kKsChunk][kKsRows + 1];     // +1: the transposing store hits 32 banks
    int32_t out_row[kKsRows];                        // output sample of each gate, -1: none
};

// tiles[((cb * 1024 + i) * 4 + plane) * 64 + lane] = 16 bytes: byte q is plane `plane` of
// KSK[i][4 * (lane / 32) + q / 4][q % 4][32 * cb + lane % 32]  (value 0 and words past n: 0)
__global__ __launch_bounds__(256) void ksk_to_tiles_kernel(const uint32_t *__restrict__ ksk, int stride, int words,
                                                           v4i *__restrict__ tiles) {
    const int i = blockIdx.x, cb = blockIdx.y;
    const int plane = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int c = 32 * cb + (lane & 31);
    uint32_t packed[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int j = 4 * (lane >> 5) + (q >> 2), v = q & 3;
        uint32_t x = (v && c < words) ? ksk[((size_t)(i * 8 + j) * 3 + (v - 1)) * stride + c] : 0u;
        int32_t digit = 0;
#pragma unroll
        for (int b = 0; b <= 3; ++b) {
            digit = (int8_t)(x & 0xFFu);
            x = (x - (uint32_t)digit) >> 8;            // exact: the low byte is zero after the subtraction
            if (b == plane) break;
        }
        packed[q >> 2] |= ((uint32_t)digit & 0xFFu) << (8 * (q & 3));
    }
    v4i t;
    t.x = (int)packed[0]; t.y = (int)packed[1]; t.z = (int)packed[2]; t.w = (int)packed[3];
    tiles[(((size_t)cb * kN + i) * 4 + plane) * 64 + lane] = t;
}

template <bool SPLIT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void key_switch_mfma_kernel(KeySwitchArgs a) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    KsMatrixLds &lds = *reinterpret_cast<KsMatrixLds *>(lds_raw);
    uint32_t (&mask_words)[kKsChunk][kKsRows + 1] = lds.mask_words;
    int32_t (&out_row)[kKsRows] = lds.out_row;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wr = wave >> 1;                                   // which 128 gates
    const int cb = 2 * blockIdx.y + (wave & 1);                 // which 32 output words
    const size_t g0 = (size_t)blockIdx.x * kKsRows;
    const int words = a.n + 1;
    {
        const size_t gi = g0 + tid;
        int32_t row = -1;
        if (gi < a.count) {
            if (a.recs) { if (a.recs[gi].op != TFHE_MUX_ELSE) row = a.recs[gi].out; }
            else if (!a.uniform_mux) row = (int32_t)gi;
            else if (!(gi & 1)) row = (int32_t)(gi >> 1);
        }
        out_row[tid] = row;
    }
    v16i acc[4][4];
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][b][r] = 0;
    const v4i *tiles = reinterpret_cast<const v4i *>(a.ksk_tiles) + (size_t)cb * kN * 4 * 64 + lane;
    const uint32_t round = 1u << (31 - 16);
    const int byte_shift = 24 - 8 * (lane >> 5);               // digits 0..3 or 4..7 of the word
    const int my_row = wr * 128 + (lane & 31);

    // a.splits workgroups (blockIdx.z) share the 1,024 mask words of their gates: each takes a
    // contiguous range and adds its partial sum into the zeroed outputs (integer adds commute:
    // still exact).  That is what gives a small batch enough workgroups to use the whole chip.
    // (SPLIT = false: one workgroup takes them all, and every loop bound is a constant)
    const int per_split = SPLIT ? kN / a.splits : kN;           // >= 32, a multiple of kKsAhead
    const int w_begin = SPLIT ? (int)blockIdx.z * per_split : 0, w_end = w_begin + per_split;
    const int chunk = SPLIT && per_split < kKsChunk ? per_split : kKsChunk;   // a power of two
    const int chunk_shift = 31 - __builtin_clz(chunk);
    const bool wave_live = g0 + (size_t)wr * 128 < a.count;     // none of the wave's 128 gates exists otherwise

    // key tiles of the next kKsAhead mask words, in a ring of registers
    v4i ring[kKsAhead][4];
#pragma unroll
    for (int s = 0; s < kKsAhead; ++s)
#pragma unroll
        for (int b = 0; b < 4; ++b) ring[s][b] = tiles[((size_t)(w_begin + s) * 4 + b) * 64];

    for (int i0 = w_begin; i0 < w_end; i0 += chunk) {
        __syncthreads();                                        // the previous chunk has been consumed
        // consecutive lanes read consecutive mask words of one gate; a dead gate stages all-zero digits
        for (int idx = tid; idx < chunk * kKsRows; idx += 256) {
            const int g = idx >> chunk_shift, ii = idx & (chunk - 1);
            mask_words[ii][g] = out_row[g] >= 0 ? a.ext[(g0 + g) * (size_t)(kN + 1) + i0 + ii] + round : 0u;
        }
        __syncthreads();
        if (!wave_live) continue;
        for (int i1 = 0; i1 < chunk; i1 += kKsAhead) {
#pragma unroll
            for (int s = 0; s < kKsAhead; ++s) {
                const int ii = i1 + s;
#pragma unroll
                for (int rt = 0; rt < 4; ++rt) {
                    const uint32_t w = (mask_words[ii][my_row + 32 * rt] >> byte_shift) & 0xFFu;
                    v4i at;
                    at.x = (int)(1u << (((w >> 6) & 3u) << 3));
                    at.y = (int)(1u << (((w >> 4) & 3u) << 3));
                    at.z = (int)(1u << (((w >> 2) & 3u) << 3));
                    at.w = (int)(1u << ((w & 3u) << 3));
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        acc[rt][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(at, ring[s][b], acc[rt][b], 0, 0, 0);
                }
                // refill the slot with the tiles kKsAhead mask words on (the last ones reload the end)
                const int nxt = i0 + ii + kKsAhead < kN ? i0 + ii + kKsAhead : kN - 1;
#pragma unroll
                for (int b = 0; b < 4; ++b) ring[s][b] = tiles[((size_t)nxt * 4 + b) * 64];
            }
        }
    }
    // accumulator register r of lane l: row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32
    const int c = 32 * cb + (lane & 31);
    if (c < words) {
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int g = wr * 128 + 32 * rt + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int32_t row = out_row[g];
                if (row < 0) continue;
                const uint32_t sum = (uint32_t)acc[rt][0][r] + ((uint32_t)acc[rt][1][r] << 8) +
                                     ((uint32_t)acc[rt][2][r] << 16) + ((uint32_t)acc[rt][3][r] << 24);
                const uint32_t body = (c == a.n && (!SPLIT || blockIdx.z == 0)) ? a.ext[(g0 + g) * (size_t)(kN + 1) + kN] : 0u;
                if (SPLIT) atomicAdd(a.out + (size_t)row * words + c, body - sum);
                else a.out[(size_t)row * words + c] = body - sum;
            }
    }
}

// Multiplexer: the two half results (ring-key samples of AND(s,a) and AND(NOT s,b)) are summed,
// 1/8 is added to the body, and the sum is what the key switch of the first half consumes.
__global__ void mux_combine_kernel(uint32_t *ext, const tfhe_gate_rec *recs, size_t count) {
    const size_t e = blockIdx.x;
    const bool first = recs ? recs[e].op == TFHE_MUX : (e & 1) == 0;
    if (!first || e + 1 >= count) return;
    uint32_t *dst = ext + e * (size_t)(kN + 1);
    const uint32_t *add = dst + (kN + 1);
    for (int j = threadIdx.x; j <= kN; j += blockDim.x) dst[j] += add[j] + (j == kN ? kEighth : 0u);
}

// out[k] = +-wires[ref.wire]  or the noiseless sample of the constant bit
__global__ void gather_outputs_kernel(const uint32_t *wires, const tfhe_out_ref *refs, uint32_t *out,
                                      size_t count, int words) {
    const size_t k = blockIdx.x;
    if (k >= count) return;
    const tfhe_out_ref r = refs[k];
    for (int w = threadIdx.x; w < words; w += blockDim.x) {
        uint32_t v;
        if (r.wire >= 0) {
            v = wires[(size_t)r.wire * words + w];
            if (r.value) v = 0u - v;
        } else {
            v = w == words - 1 ? (r.value ? kEighth : 0u - kEighth) : 0u;
        }
        out[k * (size_t)words + w] = v;
    }
}

__global__ void fill_trivial_kernel(uint32_t *ct, int words, uint32_t body) {
    for (int w = threadIdx.x; w < words; w += blockDim.x) ct[w] = w == words - 1 ? body : 0u;
}

// Register-resident double-precision FMA loop: what the vector ALU of this device sustains when
// nothing but arithmetic is in the way (16 independent chains per lane, no memory traffic).  The
// blind rotation's achieved rate is quoted against this measured figure beside the published peak.
constexpr int kPeakChains = 16, kPeakUnroll = 8;
__global__ __launch_bounds__(256) void fp64_fma_peak_kernel(double *sink, int iters, double a, double b) {
    double v[kPeakChains];
#pragma unroll
    for (int c = 0; c < kPeakChains; ++c) v[c] = (double)(threadIdx.x + c) * 1e-9;
    for (int i = 0; i < iters; ++i)
#pragma unroll
        for (int u = 0; u < kPeakUnroll; ++u)
#pragma unroll
            for (int c = 0; c < kPeakChains; ++c) v[c] = fma(v[c], a, b);
    double total = 0.0;
#pragma unroll
    for (int c = 0; c < kPeakChains; ++c) total += v[c];
    if (total == 12345.678) sink[0] = total;       // never true: keeps the chains alive
}

}  // namespace

// Compute units of the current device (cached).
static int device_cus() {
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
            return n;
        return 0;
    }();
    return cus;
}

// Largest batch that goes to the latency variant: one gate per compute unit of the device.
static int latency_batch_limit() {
    static const int limit = [] {
        if (const char *e = getenv("TFHE_LATENCY_BATCH")) return atoi(e);
        return device_cus();
    }();
    return limit;
}

// Upper bound on the workgroups of a throughput launch, 0 = none (one workgroup per gate, the
// default).  With a bound -- three per CU is what stays resident -- each workgroup takes every
// grid-th gate and all of them walk the key rows together from the first gate to the last.
// Measured on 12,288 gates: workgroups that start together stay in the same phase of the step,
// so their transform, product and key-load phases coincide instead of overlapping, and the
// launch takes 68 ms against 56 ms with one workgroup per gate, whose start times spread out.
static int resident_groups() {
    static const int groups = [] {
        if (const char *e = getenv("TFHE_RESIDENT_GROUPS")) { const int v = atoi(e); if (v > 0) return v; }
        return 0;
    }();
    return groups;
}

// Kernels that use more than 64 KB of dynamic LDS have to be told so once per device;
// `done` is that kernel's own bit mask of devices.
static int allow_dynamic_lds(const void *kernel, size_t bytes, std::atomic<uint64_t> &done) {
    int dev = 0;
    TFHE_HIP(hipGetDevice(&dev));
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return TFHE_OK;
    TFHE_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    done.fetch_or(bit, std::memory_order_release);
    return TFHE_OK;
}

size_t blind_rotate_lds_bytes() { return sizeof(GateLds); }

// ------------------------------------------------------------------------------------------
// Scratch of the entry point that allocates nothing: the extracted samples between the blind
// rotation and the key switch of at most kStaticGates gates.  Every device the library runs on
// holds its own copy of the array at its own address, looked up once per device at key upload;
// host code only ever uses that looked-up pointer, never the array's name.
// ------------------------------------------------------------------------------------------
constexpr size_t kStaticGates = TFHE_NOALLOC_MAX_GATES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) uint32_t scratch[kStaticGates * (kN + 1)];
static std::atomic<uint32_t *> scratch_of_device[kMaxDevices];

size_t static_scratch_gates() { return kStaticGates; }

int static_scratch_init() {
    int dev = 0;
    TFHE_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return set_error(TFHE_E_HIP, "device index %d out of range", dev);
    if (scratch_of_device[dev].load(std::memory_order_acquire)) return TFHE_OK;
    uint32_t *ptr = nullptr;
    TFHE_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return set_error(TFHE_E_HIP, "no device address for the static scratch array");
    scratch_of_device[dev].store(ptr, std::memory_order_release);
    return TFHE_OK;
}

uint32_t *static_scratch_ptr() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    return scratch_of_device[dev].load(std::memory_order_acquire);
}

int launch_bk_to_spectrum(const uint32_t *bk_raw, double2 *bk_fft, const double2 *tables, int n,
                          hipStream_t stream) {
    hipLaunchKernelGGL(bk_to_spectrum_kernel, dim3((unsigned)n * 4), dim3(256), 0, stream, bk_raw, bk_fft, tables);
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

// the four blind-rotation kernels and the two matrix-core key-switch kernels, with their
// dynamic LDS sizes and per-device "attribute set" masks
namespace {
struct BigLdsKernel { const void *fn; size_t lds; std::atomic<uint64_t> done; };
BigLdsKernel big_lds_kernels[6] = {
    {reinterpret_cast<const void *>(&blind_rotate_kernel<false>), sizeof(GateLds), {0}},
    {reinterpret_cast<const void *>(&blind_rotate_kernel<true>), sizeof(GateLds), {0}},
    {reinterpret_cast<const void *>(&blind_rotate_latency_kernel<false>), sizeof(GateLds), {0}},
    {reinterpret_cast<const void *>(&blind_rotate_latency_kernel<true>), sizeof(GateLds), {0}},
    {reinterpret_cast<const void *>(&key_switch_mfma_kernel<false>), sizeof(KsMatrixLds), {0}},
    {reinterpret_cast<const void *>(&key_switch_mfma_kernel<true>), sizeof(KsMatrixLds), {0}},
};
int allow(int which) { return allow_dynamic_lds(big_lds_kernels[which].fn, big_lds_kernels[which].lds, big_lds_kernels[which].done); }
}  // namespace

// Everything a launch would otherwise set up on first use (dynamic-LDS permissions, the cached
// device properties, the address of the static scratch), done once per device at key upload so
// that later calls only launch.
int prepare_kernels() {
    (void)latency_batch_limit();
    (void)resident_groups();
    for (int k = 0; k < 6; ++k)
        if (int rc = allow(k)) return rc;
    return static_scratch_init();
}

int launch_blind_rotate(const BlindRotateArgs &a, hipStream_t stream) {
    if (a.count == 0) return TFHE_OK;
    const size_t lds = sizeof(GateLds);
    const bool latency = a.count <= (size_t)latency_batch_limit();
    if (int rc = allow((latency ? 2 : 0) + (a.margin ? 1 : 0))) return rc;
    if (latency) {
        // at most one gate per CU: the variant that requests each key row a step ahead
        const dim3 grid((unsigned)a.count);
        if (a.margin) hipLaunchKernelGGL(blind_rotate_latency_kernel<true>, grid, dim3(kThreadsPerGate), lds, stream, a);
        else hipLaunchKernelGGL(blind_rotate_latency_kernel<false>, grid, dim3(kThreadsPerGate), lds, stream, a);
    } else {
        const size_t bound = (size_t)resident_groups();
        const dim3 grid((unsigned)(bound ? std::min(a.count, bound) : a.count));
        if (a.margin) hipLaunchKernelGGL(blind_rotate_kernel<true>, grid, dim3(kThreadsPerGate), lds, stream, a);
        else hipLaunchKernelGGL(blind_rotate_kernel<false>, grid, dim3(kThreadsPerGate), lds, stream, a);
    }
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

int launch_ksk_to_tiles(const uint32_t *ksk, int stride, int words, void *tiles, hipStream_t stream) {
    hipLaunchKernelGGL(ksk_to_tiles_kernel, dim3(kN, 16), dim3(256), 0, stream, ksk, stride, words,
                       reinterpret_cast<v4i *>(tiles));
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

size_t ksk_tiles_bytes() { return (size_t)16 * kN * 4 * 64 * sizeof(v4i); }

int launch_key_switch(const KeySwitchArgs &a, hipStream_t stream) {
    if (a.count == 0) return TFHE_OK;
    if (a.ksk_tiles && a.matrix && a.t == 8 && a.basebit == 2 && a.n + 1 <= 512) {
        // fewer than one workgroup per CU: share each gate's mask words between workgroups
        KeySwitchArgs m = a;
        const unsigned row_blocks = (unsigned)((a.count + kKsRows - 1) / kKsRows);
        m.splits = 1;
        while (m.splits < 32 && row_blocks * 8 * m.splits < 256) m.splits *= 2;
        if (int rc = allow(m.splits > 1 ? 5 : 4)) return rc;
        if (m.splits > 1) {
            hipLaunchKernelGGL(zero_outputs_kernel, dim3((unsigned)a.count), dim3(256), 0, stream, m);
            TFHE_HIP(hipGetLastError());
        }
        const dim3 grid(row_blocks, 8, (unsigned)m.splits);
        if (m.splits > 1)
            hipLaunchKernelGGL(key_switch_mfma_kernel<true>, grid, dim3(256), sizeof(KsMatrixLds), stream, m);
        else
            hipLaunchKernelGGL(key_switch_mfma_kernel<false>, grid, dim3(256), sizeof(KsMatrixLds), stream, m);
        TFHE_HIP(hipGetLastError());
        return TFHE_OK;
    }
    if (a.splits < 1 || (a.splits & (a.splits - 1)) || a.splits > 64)
        return set_error(TFHE_E_PARAM, "key-switch splits must be a power of two <= 64");
    if (a.splits > 1) {
        hipLaunchKernelGGL(zero_outputs_kernel, dim3((unsigned)a.count), dim3(256), 0, stream, a);
        TFHE_HIP(hipGetLastError());
    }
    const dim3 grid((unsigned)(a.count * a.splits)), block(256);
    switch (a.t) {
#define KS_CASE(T) case T: hipLaunchKernelGGL(key_switch_kernel<T>, grid, block, 0, stream, a); break;
        KS_CASE(1) KS_CASE(2) KS_CASE(3) KS_CASE(4) KS_CASE(5) KS_CASE(6) KS_CASE(7) KS_CASE(8)
        KS_CASE(9) KS_CASE(10) KS_CASE(11) KS_CASE(12)
#undef KS_CASE
    default: return set_error(TFHE_E_PARAM, "unsupported key-switch digit count %d", a.t);
    }
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

int launch_mux_combine(uint32_t *ext, const tfhe_gate_rec *recs, size_t count, hipStream_t stream) {
    if (count == 0) return TFHE_OK;
    hipLaunchKernelGGL(mux_combine_kernel, dim3((unsigned)count), dim3(256), 0, stream, ext, recs, count);
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

int launch_gather_outputs(const uint32_t *wires, const tfhe_out_ref *refs, uint32_t *out, size_t count,
                          int words, hipStream_t stream) {
    if (count == 0) return TFHE_OK;
    hipLaunchKernelGGL(gather_outputs_kernel, dim3((unsigned)count), dim3(256), 0, stream, wires, refs, out,
                       count, words);
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

// Time the FMA loop with HIP events on `stream`; *tflops = achieved double-precision rate.
int measure_fp64_fma_peak(hipStream_t stream, double *sink, double *tflops) {
    const int cus = device_cus() > 0 ? device_cus() : 256;
    const int blocks = cus * 8, iters = 4096;               // 8 workgroups of 4 waves per CU: 8 waves per SIMD
    hipEvent_t t0, t1;
    TFHE_HIP(hipEventCreate(&t0));
    TFHE_HIP(hipEventCreate(&t1));
    float best = 0.0f;
    int rc = TFHE_OK;
    for (int rep = 0; rep < 3 && rc == TFHE_OK; ++rep) {      // the first launch warms the clocks up
        hipError_t e = hipEventRecord(t0, stream);
        hipLaunchKernelGGL(fp64_fma_peak_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, sink, iters, 0.999999, 1e-7);
        if (e == hipSuccess) e = hipGetLastError();
        if (e == hipSuccess) e = hipEventRecord(t1, stream);
        if (e == hipSuccess) e = hipEventSynchronize(t1);
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t0, t1);
        if (e != hipSuccess) { rc = set_error(TFHE_E_HIP, "FMA peak measurement failed: %s", hipGetErrorString(e)); break; }
        if (rep == 0 || ms < best) best = ms;
    }
    (void)hipEventDestroy(t0);
    (void)hipEventDestroy(t1);
    if (rc) return rc;
    const double flops = 2.0 * kPeakChains * kPeakUnroll * (double)iters * 256.0 * (double)blocks;
    *tflops = flops / ((double)best * 1e-3) / 1e12;
    return TFHE_OK;
}

int launch_fill_trivial(uint32_t *ct, int words, int bit, hipStream_t stream) {
    hipLaunchKernelGGL(fill_trivial_kernel, dim3(1), dim3(256), 0, stream, ct, words,
                       bit ? kEighth : 0u - kEighth);
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

}  // namespace tfhe
