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

// Forward transform of the 8 folded points held in x; leaves the spectrum in buf in
// slot order (slot = 64 * register + lane).
__device__ __forceinline__ void forward_to_slots(double2 (&x)[8], const Lane &ln, double2 *buf, int L) {
    fwd_pass1_store(x, ln, buf, L);
    wave_sync();
    fwd_pass2_load(x, buf, L);
    wave_sync();
    fwd_pass2_store(x, ln, buf, L);
    wave_sync();
    fwd_pass3(x, buf, L);
    wave_sync();
#pragma unroll
    for (int k = 0; k < 8; ++k) buf[k * 64 + L] = x[k];
}

// Inverse transform of the spectrum held in buf (slot order); x[m] is 512 times the folded
// point L + 64 m (real part: coefficient L + 64 m, imaginary part: coefficient L + 64 m + 512).
__device__ __forceinline__ void inverse_from_slots(double2 (&x)[8], const Lane &ln, double2 *buf, int L) {
#pragma unroll
    for (int k = 0; k < 8; ++k) x[k] = buf[k * 64 + L];
    wave_sync();
    inv_pass3_store(x, ln, buf, L);
    wave_sync();
    inv_pass2(x, buf, L);
    wave_sync();
    inv_pass2_store(x, buf, L);
    wave_sync();
    inv_pass1(x, ln, buf, L);
}

// ------------------------------------------------------------------------------------------
// Bootstrapping key -> transform domain.  One wave per (sample row, component, limb).
// bk_raw [n][4][2][1024] uint32  ->  bk_fft [n][4][o = 2*component + limb][512] complex.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void bk_to_spectrum_kernel(const uint32_t *__restrict__ bk_raw,
                                                            double2 *__restrict__ bk_fft,
                                                            const double2 *__restrict__ tables) {
    __shared__ double2 buf[kBufWords];
    const int L = threadIdx.x;
    const int limb = blockIdx.x & 1;
    const size_t poly = blockIdx.x >> 1;           // (i * 4 + r) * 2 + c
    const int c = (int)(poly & 1);
    const size_t row = poly >> 1;                  // i * 4 + r
    const uint32_t *src = bk_raw + poly * kN;
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
    forward_to_slots(x, ln, buf, L);
    wave_sync();
    double2 *dst = bk_fft + (row * 4 + (size_t)(c * 2 + limb)) * kHalf;
#pragma unroll
    for (int k = 0; k < 8; ++k) dst[k * 64 + L] = buf[k * 64 + L];
}

// ------------------------------------------------------------------------------------------
// Blind rotation of B gates per workgroup, 256 threads (4 waves) per gate.
//   prologue  c = (0, kappa) + m (s0 c0 + s1 c1); abar_j = round(c_j * 2N / 2^32); ACC = (0, X^-bbar v)
//   n steps   D = X^abar_i ACC - ACC; 4 digit polynomials -> 4 forward FFTs (wave r);
//             products with the transform-domain key row (all threads, one key load shared by the
//             B gates); 4 inverse FFTs (wave o = component, limb); ACC += rounded results
//   epilogue  sample extraction of coefficient 0 -> ext[gate][1025]
// ------------------------------------------------------------------------------------------
struct GateLds {
    double2 spec[4][kBufWords];   // per wave: FFT scratch, then spectrum / product in slot order
    uint32_t acc[2][kN];          // accumulator (mask, body), stored bitwise complemented: ~ACC = -ACC - 1
    uint16_t bar[1032];           // abar_0 .. abar_{n-1}, bbar
};
// the rotation or-s a masked offset into the accumulator's address when that is 4 KB aligned
static_assert(offsetof(GateLds, acc) % (kN * sizeof(uint32_t)) == 0, "accumulator at a multiple of 4 KB");

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

// (x & mask) | y in one instruction; mask is wave-uniform
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t y) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask), "v"(y));
    return r;
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

// AHEAD: how many of the step's key-load parts (a part = 8 values = 32 registers; a step of a
// one-gate workgroup has 4) are loaded for step i + 1 as soon as the products of step i are
// done, so that their latency hides behind the inverse transforms, the rotation and the
// forward transforms.  All of them only for launches that leave one workgroup per CU; at full
// occupancy other workgroups already cover that latency (one part ahead: no measurable gain).
// TPG: threads per gate, 256 or 512.  The transforms, the rotation and the accumulation are the
// work of four waves; with 512 threads the other four waves only take their share of the
// spectral products (one slot per thread instead of two), which shortens a lone gate's step.
template <int B, bool MARGIN, int AHEAD, int TPG = kThreadsPerGate>
__device__ __forceinline__ void blind_rotate_body(const BlindRotateArgs &a) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    GateLds *lds = reinterpret_cast<GateLds *>(lds_raw);

    const int tid = threadIdx.x;
    static_assert(TPG == 256 || TPG == 512, "four or eight waves per gate");
    const int g = tid / TPG;               // gate slot in this workgroup
    const int lt = tid % TPG;              // thread within the gate
    const int wv = lt >> 6;                // wave within the gate
    const bool fft_wave = TPG == 256 || wv < 4;    // wave-uniform
    const int L = tid & 63;
    GateLds &my = lds[g];
    const size_t gi = (size_t)blockIdx.x * B + g;
    const bool live = gi < a.count;

    Lane ln;
    lane_init(ln, a.tables, L);
    const __amdgpu_buffer_rsrc_t key_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<double2 *>(a.bk_fft), 0, (int)((size_t)a.n * 16 * kHalf * sizeof(double2)), 0x00020000);

    // ---- prologue ----
    {
        int op = a.uniform_op;
        size_t i0 = gi, i1 = gi;
        uint32_t s0 = 1u, s1 = 1u;
        const uint32_t *src1 = a.in1;
        if (live && a.recs) {
            const tfhe_gate_rec r = a.recs[gi];
            op = r.op; i0 = (size_t)r.in0; i1 = (size_t)r.in1;
            s0 = r.neg0 ? 0xFFFFFFFFu : 1u; s1 = r.neg1 ? 0xFFFFFFFFu : 1u;
        } else if (live && op == TFHE_MUX) {
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
        for (int j = lt; j <= a.n; j += TPG) {
            uint32_t c = 0;
            if (live) {
                c = mult * (s0 * a.in0[i0 * w + j] + s1 * src1[i1 * w + j]);
                if (j == a.n) c += kappa;
            }
            my.bar[j] = (uint16_t)(((c + (1u << 20)) >> 21) & 2047u);
        }
    }
    __syncthreads();
    {
        const int bbar = my.bar[a.n];
        const int bb = bbar & (kN - 1);
        const uint32_t first = bbar < kN ? kEighth : 0u - kEighth;   // X^-bbar v, closed form
        for (int j = lt; j < kN; j += TPG) {
            my.acc[0][j] = ~0u;
            my.acc[1][j] = ~(j < kN - bb ? first : 0u - first);
        }
    }
    __syncthreads();

    const int comp = (wv & 3) >> 1;             // forward: component of D; inverse: component of ACC
    const int sel = wv & 1;                     // forward: digit index; inverse: limb
    // Signed digit `sel` of x: add the rounding constant and the half-bases of the lower digits
    // (not its own: its two's-complement field then already is the centred digit), move the
    // field to the top of the word, shift back down arithmetically.
    const uint32_t dround = 1u << (31 - 2 * a.bgbit);
    const uint32_t doffset = sel ? dround : dround + (1u << (31 - a.bgbit));
    const uint32_t dfield = (uint32_t)(32 - a.bgbit * (1 + sel));   // lowest bit of the digit's field
    double worst = 0.0;

    constexpr int kSlotsPerThread = (kHalf + TPG * B - 1) / (TPG * B);
    static_assert(AHEAD >= 0 && AHEAD <= 2 * kSlotsPerThread, "parts of one step");
    double2 ahead[AHEAD ? AHEAD : 1][4][2];     // [part = 2 * pass + half][row][output]
    auto load_ahead = [&](int row) {
        const uint32_t row_bytes = (uint32_t)row * 16u * kHalf * (uint32_t)sizeof(double2);
#pragma unroll
        for (int part = 0; part < AHEAD; ++part)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int o = 0; o < 2; ++o)
                    ahead[part][r][o] = load_key(
                        key_rsrc, (uint32_t)(tid + (part >> 1) * TPG * B) * (uint32_t)sizeof(double2),
                        row_bytes + (uint32_t)((r * 4 + 2 * (part & 1) + o) * kHalf * sizeof(double2)));
    };
    if (AHEAD) load_ahead(0);

    int abar_next = my.bar[0];
    for (int i = 0; i < a.n; ++i) {
        double2 x[8];
        if (fft_wave) {
        // ---- rotate, subtract, decompose, fold and twist ----
        // read one step ahead (off the critical path); the same in every lane, so it goes to a scalar
        // register and the per-coefficient offsets below are scalar arithmetic
        const int abar = __builtin_amdgcn_readfirstlane(abar_next);
        // LDS address of the component's accumulator as an integer: 4 KB aligned when the workgroup holds
        // one gate (dynamic LDS starts at 0), so that a masked offset can be or-ed in
        typedef __attribute__((address_space(3))) const uint32_t lds_word;
        const uint32_t acc_at = (uint32_t)(uintptr_t)(lds_word *)my.acc[comp];
        const uint32_t lane4 = (uint32_t)L << 2;
        const uint32_t back4 = (uint32_t)(0 - abar) << 2;       // X^abar reads abar coefficients back, mod 8192 bytes
        // per coefficient: byte offset of its source = lane part + scalar part (kept on the scalar ALU)
        uint32_t shift4[8][2];
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                // + 4096: bit 12 of the sum then says "source not past X^N"
                shift4[m][h] = back4 + (uint32_t)(64 * m + h * kHalf) * 4u + 4096u;
                asm("" : "+s"(shift4[m][h]));
            }
        // all sixteen rotated reads are issued before any of them is consumed
        uint32_t rot[8][2];
        if ((acc_at & 4095u) == 0) {              // wave-uniform; true for one gate per workgroup
#pragma unroll
            for (int m = 0; m < 8; ++m)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    rot[m][h] = *(lds_word *)(uintptr_t)and_or(lane4 + shift4[m][h], 4092u, acc_at);
        } else {
#pragma unroll
            for (int m = 0; m < 8; ++m)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    rot[m][h] = *(lds_word *)(uintptr_t)(((lane4 + shift4[m][h]) & 4092u) + acc_at);
        }
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            int32_t dig[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int j = L + 64 * m + h * kHalf;
                const uint32_t src = lane4 + shift4[m][h];
                // With ACC stored as c = ~ACC, the step's  +-ACC[src] - ACC[j] + doffset  is
                //   source not past X^N:  -c[src] + c[j] + doffset = (c[src] ^ ~0) + c[j] + doffset + 1
                //   source past X^N:       c[src] + c[j] + doffset + 2
                // i.e. (c[src] ^ flip) + c[j] + (doffset + 2 + flip) with flip = ~0 or 0: four instructions.
                const uint32_t flip = (uint32_t)__builtin_amdgcn_sbfe((int32_t)src, 12u, 1u);
                const uint32_t d = (rot[m][h] ^ flip) + my.acc[comp][j] + (doffset + 2u + flip);
                dig[h] = __builtin_amdgcn_sbfe((int32_t)d, dfield, (uint32_t)a.bgbit);    // signed field
            }
            x[m] = make_double2((double)dig[0], (double)dig[1]);
        }
        forward_to_slots(x, ln, my.spec[wv & 3], L);
        }
        __syncthreads();
        // The short phase between the two barriers starts with the key loads: waves in it go first
        // (measured: 3 % faster than equal priorities; raising it in other phases loses).
        __builtin_amdgcn_s_setprio(2);

        // ---- products with the key row: thread <-> slot, all gates of the workgroup ----
        {
            // key row i through a buffer descriptor: scalar base and row offset, 32-bit lane offset
            const uint32_t row_bytes = (uint32_t)i * 16u * kHalf * (uint32_t)sizeof(double2);
#pragma unroll
            for (int pass = 0; pass < kSlotsPerThread; ++pass) {
                const int s = tid + pass * TPG * B;
                if (TPG * B * kSlotsPerThread != kHalf && s >= kHalf) break;
                const uint32_t voff = (uint32_t)s * (uint32_t)sizeof(double2);   // uniform base + 32-bit offset
                double2 d[B][4];
#pragma unroll
                for (int q = 0; q < B; ++q)
#pragma unroll
                    for (int r = 0; r < 4; ++r) d[q][r] = lds[q].spec[r][s];
                // two outputs at a time keeps the key values of one pass in 32 registers
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    double2 k[4][2];
#pragma unroll
                    for (int r = 0; r < 4; ++r)
#pragma unroll
                        for (int o = 0; o < 2; ++o)
                            k[r][o] = 2 * pass + half < AHEAD
                                          ? ahead[2 * pass + half < AHEAD ? 2 * pass + half : 0][r][o]
                                          : load_key(key_rsrc, voff, row_bytes + (uint32_t)((r * 4 + 2 * half + o) *
                                                                                                 kHalf * sizeof(double2)));
#pragma unroll
                    for (int q = 0; q < B; ++q)
#pragma unroll
                        for (int o = 0; o < 2; ++o) {
                            // fused multiply-adds, two independent chains per part
                            double yr = d[q][0].x * k[0][o].x, yi = d[q][0].x * k[0][o].y;
                            double zr = -d[q][0].y * k[0][o].y, zi = d[q][0].y * k[0][o].x;
#pragma unroll
                            for (int r = 1; r < 4; ++r) {
                                yr = fma(d[q][r].x, k[r][o].x, yr);
                                yi = fma(d[q][r].x, k[r][o].y, yi);
                                zr = fma(-d[q][r].y, k[r][o].y, zr);
                                zi = fma(d[q][r].y, k[r][o].x, zi);
                            }
                            yr += zr; yi += zi;
                            lds[q].spec[2 * half + o][s] = make_double2(yr, yi);
                        }
                }
            }
        }
        __syncthreads();
        __builtin_amdgcn_s_setprio(0);
        if (AHEAD) load_ahead(i + 1 < a.n ? i + 1 : i);
        abar_next = my.bar[i + 1];           // bar[n] exists (it holds bbar)

        // ---- inverse transform, exact rounding, accumulate ----
        if (fft_wave) {
        inverse_from_slots(x, ln, my.spec[wv & 3], L);
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
                atomicAdd(&my.acc[comp][L + 64 * m + h * kHalf], r);
            }
        }
        }
        __syncthreads();
    }

    // ---- epilogue: the constant coefficient as an LWE sample under the ring key ----
    if (live) {
        uint32_t *ext = a.ext + gi * (size_t)(kN + 1);
        // ACC = ~c, -ACC = c + 1
        for (int j = lt; j < kN; j += TPG) ext[j] = j == 0 ? ~my.acc[0][0] : my.acc[0][kN - j] + 1u;
        if (lt == 0) ext[kN] = ~my.acc[1][0];
    }
    if (MARGIN) {
        // non-negative doubles order like their bit patterns
        atomicMax(reinterpret_cast<unsigned long long *>(a.margin),
                  (unsigned long long)__double_as_longlong(worst));
    }
}

template <int B, bool MARGIN>
__global__ __launch_bounds__(kThreadsPerGate *B) __attribute__((amdgpu_waves_per_eu(3, 3))) void blind_rotate_kernel(BlindRotateArgs a) {
    blind_rotate_body<B, MARGIN, 0>(a);
}

// The same step for batches of at most one gate per CU, where a gate's latency is all that counts.
constexpr int kLatencyThreads = 512;
template <bool MARGIN>
__global__ __launch_bounds__(kLatencyThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void blind_rotate_latency_kernel(BlindRotateArgs a) {
    blind_rotate_body<1, MARGIN, 2, kLatencyThreads>(a);
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
// Key switch, G gates per workgroup (the fast path for t = 8 digits in base 4, n + 1 <= 512).
// Every key row is loaded once per workgroup and subtracted from the gates whose digit selects
// it, so the key traffic per gate is 1/G of the one-gate-per-workgroup kernel.  Thread p owns the
// adjacent output words 2p, 2p+1 of all G gates.  For one (mask word i, digit position j) each
// wave parks its 128-word slice of the three rows in a private LDS table whose row 0 stays
// zero; a gate's digit is uniform over the workgroup, so the gate picks its row with a uniform
// LDS offset -- the LDS does the gather.  The rounded mask words of the G gates are staged
// through LDS 64 at a time.
// ------------------------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(256) void key_switch_shared_kernel(KeySwitchArgs a) {
    constexpr int T = 8, kChunk = 64;
    __shared__ uint32_t mask_words[kChunk][G];
    __shared__ uint2 stage[4][4][64];             // [wave][digit value][lane]
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const size_t g0 = (size_t)blockIdx.x * G;
    const int words = a.n + 1;
    const bool owner = 2 * tid < words;            // 2p+1 may be the zero padding word of a row
    const int pair = owner ? tid : 0;              // idle threads shadow pair 0 and store nothing

    // an item is live if it exists and is not the second half of a multiplexer
    auto is_live = [&](size_t gi) {
        if (gi >= a.count) return false;
        return a.recs ? a.recs[gi].op != TFHE_MUX_ELSE : !(a.uniform_mux && (gi & 1));
    };
    uint2 acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const bool live = is_live(g0 + g);
        const uint32_t body = live ? a.ext[(g0 + g) * (size_t)(kN + 1) + kN] : 0u;
        acc[g].x = 2 * pair == a.n ? body : 0u;
        acc[g].y = 2 * pair + 1 == a.n ? body : 0u;
    }
    stage[wave][0][lane] = make_uint2(0u, 0u);
    const uint32_t round = 1u << (31 - T * 2);
    const unsigned char *table = reinterpret_cast<const unsigned char *>(&stage[wave][0][lane]);
    for (int i0 = 0; i0 < kN; i0 += kChunk) {
        __syncthreads();
        for (int idx = tid; idx < kChunk * G; idx += 256) {
            const int g = idx / kChunk, ii = idx % kChunk;
            const bool live = is_live(g0 + g);
            mask_words[ii][g] = live ? a.ext[(g0 + g) * (size_t)(kN + 1) + i0 + ii] + round : 0u;
        }
        __syncthreads();
        for (int ii = 0; ii < kChunk; ++ii) {
            const uint32_t *rows = a.ksk + (size_t)(i0 + ii) * T * 3 * a.stride;
            uint2 r[T][3];
#pragma unroll
            for (int j = 0; j < T; ++j)
#pragma unroll
                for (int v = 0; v < 3; ++v)
                    r[j][v] = *reinterpret_cast<const uint2 *>(rows + (size_t)(j * 3 + v) * a.stride + 2 * pair);
            uint32_t ai[G];
#pragma unroll
            for (int g = 0; g < G; ++g) ai[g] = __builtin_amdgcn_readfirstlane(mask_words[ii][g]);
#pragma unroll
            for (int j = 0; j < T; ++j) {
                wave_sync();                       // the previous table has been read by every lane
#pragma unroll
                for (int v = 0; v < 3; ++v) stage[wave][v + 1][lane] = r[j][v];
                wave_sync();
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const uint32_t v = (ai[g] >> (30 - 2 * j)) & 3u;
                    const uint2 sub = *reinterpret_cast<const uint2 *>(table + v * (64 * sizeof(uint2)));
                    acc[g].x -= sub.x;
                    acc[g].y -= sub.y;
                }
            }
        }
    }
    if (owner) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (is_live(g0 + g)) {
                const size_t out_index =
                    a.recs ? (size_t)a.recs[g0 + g].out : (a.uniform_mux ? (g0 + g) >> 1 : g0 + g);
                uint32_t *out = a.out + out_index * (size_t)words;
                out[2 * pair] = acc[g].x;
                if (2 * pair + 1 < words) out[2 * pair + 1] = acc[g].y;
            }
        }
    }
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

}  // namespace

// Largest batch that goes to the latency variant: one gate per compute unit of the device.
static int latency_batch_limit() {
    static const int limit = [] {
        if (const char *e = getenv("TFHE_LATENCY_BATCH")) return atoi(e);
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
            return cus;
        return 0;
    }();
    return limit;
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

size_t blind_rotate_lds_bytes(int gates_per_group) { return sizeof(GateLds) * (size_t)gates_per_group; }

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
    const unsigned blocks = (unsigned)n * 4 * 2 * 2;
    hipLaunchKernelGGL(bk_to_spectrum_kernel, dim3(blocks), dim3(64), 0, stream, bk_raw, bk_fft, tables);
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

template <int B>
static int launch_br(const BlindRotateArgs &a, hipStream_t stream) {
    const size_t lds = blind_rotate_lds_bytes(B);
    static std::atomic<uint64_t> plain{0}, with_margin{0};
    if (int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&blind_rotate_kernel<B, false>), lds, plain)) return rc;
    if (int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&blind_rotate_kernel<B, true>), lds, with_margin)) return rc;
    const unsigned blocks = (unsigned)((a.count + B - 1) / B);
    if (a.margin)
        hipLaunchKernelGGL((blind_rotate_kernel<B, true>), dim3(blocks), dim3(kThreadsPerGate * B), lds, stream, a);
    else
        hipLaunchKernelGGL((blind_rotate_kernel<B, false>), dim3(blocks), dim3(kThreadsPerGate * B), lds, stream, a);
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

// Batches that leave at most one gate per CU: the variant that loads each key row a step ahead.
static int launch_br_latency(const BlindRotateArgs &a, hipStream_t stream) {
    const size_t lds = blind_rotate_lds_bytes(1);
    static std::atomic<uint64_t> plain{0}, with_margin{0};
    if (int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&blind_rotate_latency_kernel<false>), lds, plain)) return rc;
    if (int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&blind_rotate_latency_kernel<true>), lds, with_margin)) return rc;
    if (a.margin)
        hipLaunchKernelGGL(blind_rotate_latency_kernel<true>, dim3((unsigned)a.count), dim3(kLatencyThreads), lds, stream, a);
    else
        hipLaunchKernelGGL(blind_rotate_latency_kernel<false>, dim3((unsigned)a.count), dim3(kLatencyThreads), lds, stream, a);
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

int launch_blind_rotate(const BlindRotateArgs &a, int gates_per_group, hipStream_t stream) {
    if (a.count == 0) return TFHE_OK;
    if (gates_per_group == 1 && a.count <= (size_t)latency_batch_limit()) return launch_br_latency(a, stream);
    switch (gates_per_group) {
    case 1: return launch_br<1>(a, stream);
    case 2: return launch_br<2>(a, stream);
    case 3: return launch_br<3>(a, stream);
    default: return set_error(TFHE_E_PARAM, "unsupported gates per workgroup %d", gates_per_group);
    }
}

// Everything a launch would otherwise set up on first use (dynamic-LDS permissions, the cached
// device properties), done once per device at key upload so that later calls only launch.
int prepare_kernels() {
    (void)latency_batch_limit();
    const size_t lds = blind_rotate_lds_bytes(1);
    static std::atomic<uint64_t> unused[6];
    const void *kernels[6] = {reinterpret_cast<const void *>(&blind_rotate_kernel<1, false>),
                              reinterpret_cast<const void *>(&blind_rotate_kernel<1, true>),
                              reinterpret_cast<const void *>(&blind_rotate_latency_kernel<false>),
                              reinterpret_cast<const void *>(&blind_rotate_latency_kernel<true>),
                              reinterpret_cast<const void *>(&key_switch_mfma_kernel<false>),
                              reinterpret_cast<const void *>(&key_switch_mfma_kernel<true>)};
    for (int k = 0; k < 6; ++k)
        if (int rc = allow_dynamic_lds(kernels[k], k < 4 ? lds : sizeof(KsMatrixLds), unused[k])) return rc;
    return static_scratch_init();
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
        static std::atomic<uint64_t> whole{0}, split{0};
        if (int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&key_switch_mfma_kernel<false>), sizeof(KsMatrixLds), whole))
            return rc;
        if (int rc = allow_dynamic_lds(reinterpret_cast<const void *>(&key_switch_mfma_kernel<true>), sizeof(KsMatrixLds), split))
            return rc;
        // fewer than one workgroup per CU: share each gate's mask words between workgroups
        KeySwitchArgs m = a;
        const unsigned row_blocks = (unsigned)((a.count + kKsRows - 1) / kKsRows);
        m.splits = 1;
        while (m.splits < 32 && row_blocks * 8 * m.splits < 256) m.splits *= 2;
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
    if (a.t == 8 && a.basebit == 2 && a.n + 1 <= 512 && a.group > 1) {
        // more gates per workgroup = less key traffic per gate but fewer, longer workgroups
#define KS_SHARED(G)                                                                                   \
    hipLaunchKernelGGL(key_switch_shared_kernel<G>, dim3((unsigned)((a.count + G - 1) / G)), dim3(256), 0, \
                       stream, a)
        if (a.group >= 16) KS_SHARED(16);
        else if (a.group >= 8) KS_SHARED(8);
        else KS_SHARED(4);
#undef KS_SHARED
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

int launch_fill_trivial(uint32_t *ct, int words, int bit, hipStream_t stream) {
    hipLaunchKernelGGL(fill_trivial_kernel, dim3(1), dim3(256), 0, stream, ct, words,
                       bit ? kEighth : 0u - kEighth);
    TFHE_HIP(hipGetLastError());
    return TFHE_OK;
}

}  // namespace tfhe
