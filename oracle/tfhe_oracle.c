/*
 * tfhe_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-purpose CPU implementation of bootstrapped binary
 * gates on LWE ciphertexts over the 32-bit torus (the gate primitive that the
 * TAPAS paper takes from CGGI, Sec. 3.1.2 "Encrypted Prediction with FHE", and
 * uses in Sec. 4.1 "Binary OPs").  The paper treats the gate as a black box;
 * the construction written out here is the public CGGI one: gate
 * pre-combination, modulus switch, blind rotation by TRGSW external products
 * over Z_{2^32}[X]/(X^N+1), sample extraction, LWE key switching.
 *
 * All arithmetic is exact integer arithmetic modulo 2^32 on uint32_t (wrap-around
 * is the definition, not an accident).  Polynomial products are the textbook
 * negacyclic convolution, written three ways (index-by-index definition,
 * schoolbook-then-fold, Karatsuba-then-fold) so that they can be checked against
 * each other.  Nothing here is blocked, fused or reordered for speed beyond that.
 *
 * Only tests, the smoke check and the cpu_baseline leg of the benchmark may load
 * this file's library.  The GPU library shares no code with it.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef uint32_t torus32;

typedef struct {
    int32_t n;              /* LWE dimension */
    int32_t N;              /* ring degree, power of two */
    int32_t k;              /* TRLWE mask count, must be 1 */
    int32_t bk_l;           /* gadget length */
    int32_t bk_Bgbit;       /* log2 of gadget base */
    int32_t ks_t;           /* key-switch digits */
    int32_t ks_basebit;     /* log2 of key-switch base */
    int32_t lwe_noise_log2; /* stdev of fresh LWE / KSK noise = 2^this (torus units) */
    int32_t bk_noise_log2;  /* stdev of bootstrapping-key noise */
} orc_params;

/* ------------------------------------------------------------------ */
/* Counter-based random numbers: SplitMix64 (Steele, Lea, Flood 2014). */
/* The k-th output (k = 1, 2, ...) of a SplitMix64 generator whose     */
/* state starts at s is mix(s + k * GOLDEN).  A (seed, domain) pair    */
/* selects a stream: domain 0 is the generator seeded with `seed`      */
/* itself; domain d >= 1 is the generator seeded with the d-th output  */
/* of that one.                                                        */
/* ------------------------------------------------------------------ */
#define ORC_GOLDEN 0x9E3779B97F4A7C15ULL

static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

uint64_t orc_stream_key(uint64_t seed, uint32_t domain)
{
    if (domain == 0) return seed;
    return mix64(seed + (uint64_t)domain * ORC_GOLDEN);
}

uint64_t orc_rand(uint64_t seed, uint32_t domain, uint64_t index)
{
    return mix64(orc_stream_key(seed, domain) + (index + 1) * ORC_GOLDEN);
}

static uint32_t rand_u32(uint64_t seed, uint32_t domain, uint64_t index)
{
    return (uint32_t)(orc_rand(seed, domain, index) >> 32);
}

/* stream domains */
enum { D_RAW = 0, D_LWE_SK = 1, D_TRLWE_SK = 2, D_BK_A = 3, D_BK_E = 4,
       D_KSK_A = 5, D_KSK_E = 6, D_ENC_A = 7, D_ENC_E = 8 };

/*
 * Integer-only bell-shaped noise: the sum of 12 uniform 32-bit draws minus its
 * mean (Irwin-Hall) has standard deviation exactly 2^32; dividing by 2^s with
 * round-half-up gives standard deviation 2^(32-s) torus units, i.e. 2^-s as a
 * real torus element.  Draw j of sample `index` is stream element 12*index + j.
 */
int64_t orc_noise(uint64_t seed, uint32_t domain, uint64_t index, int noise_log2)
{
    int s = -noise_log2;
    if (s >= 40 || s < 1) return 0;          /* |G| < 6*2^32 < 2^35: rounds to 0 */
    int64_t G = 0;
    for (int j = 0; j < 12; ++j) G += (int64_t)rand_u32(seed, domain, 12 * index + j);
    G -= (int64_t)6 << 32;
    int64_t x = G + ((int64_t)1 << (s - 1));
    /* floor(x / 2^s) written without relying on the shift of a negative value */
    if (x >= 0) return x >> s;
    return -(((-x) + (((int64_t)1 << s) - 1)) >> s);
}

/* ------------------------------------------------------------------ */
/* Negacyclic products  c = a * b  in  Z_{2^32}[X] / (X^N + 1)          */
/* ------------------------------------------------------------------ */

/* The definition, one output index at a time: X^N = -1. */
void orc_negacyclic_definition(const uint32_t *a, const uint32_t *b, uint32_t *c, int N)
{
    for (int k = 0; k < N; ++k) {
        uint32_t acc = 0;
        for (int i = 0; i < N; ++i) {
            int j = k - i;
            if (j >= 0) acc += a[i] * b[j];
            else        acc -= a[i] * b[j + N];
        }
        c[k] = acc;
    }
}

static void fold_negacyclic(const uint32_t *lin, uint32_t *c, int N)
{
    for (int k = 0; k < N; ++k) c[k] = lin[k];
    for (int k = N; k < 2 * N - 1; ++k) c[k - N] -= lin[k];
}

/* linear (non-wrapping) product, 2n-1 coefficients, schoolbook */
__attribute__((target_clones("avx512f", "avx2", "default")))
static void linear_schoolbook(const uint32_t *restrict a, const uint32_t *restrict b,
                              uint32_t *restrict out, int n)
{
    for (int k = 0; k < 2 * n - 1; ++k) out[k] = 0;
    for (int i = 0; i < n; ++i) {
        uint32_t ai = a[i];
        uint32_t *o = out + i;
        for (int j = 0; j < n; ++j) o[j] += ai * b[j];
    }
}

void orc_negacyclic_schoolbook(const uint32_t *a, const uint32_t *b, uint32_t *c, int N)
{
    uint32_t *lin = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(2 * N));
    linear_schoolbook(a, b, lin, N);
    fold_negacyclic(lin, c, N);
    free(lin);
}

/*
 * Karatsuba on the linear product (valid in any commutative ring, here Z_{2^32}):
 * with a = a0 + X^h a1, b = b0 + X^h b1,
 *   a*b = a0b0 + X^h[(a0+a1)(b0+b1) - a0b0 - a1b1] + X^{2h} a1b1.
 * `out` receives 2n-1 coefficients; `tmp` needs 4n words.
 */
#define KARA_BASE 128
static void linear_karatsuba(const uint32_t *a, const uint32_t *b, uint32_t *out, int n, uint32_t *tmp)
{
    if (n <= KARA_BASE || (n & 1)) { linear_schoolbook(a, b, out, n); return; }
    int h = n / 2;
    uint32_t *sa = tmp, *sb = tmp + h, *mid = tmp + 2 * h, *rest = tmp + 4 * h;
    for (int i = 0; i < h; ++i) { sa[i] = a[i] + a[i + h]; sb[i] = b[i] + b[i + h]; }
    linear_karatsuba(sa, sb, mid, h, rest);                 /* (a0+a1)(b0+b1): 2h-1 */
    linear_karatsuba(a, b, out, h, rest);                   /* a0b0 -> out[0..2h-2] */
    out[2 * h - 1] = 0;
    linear_karatsuba(a + h, b + h, out + 2 * h, h, rest);   /* a1b1 -> out[2h..4h-2] */
    for (int i = 0; i < 2 * h - 1; ++i) mid[i] -= out[i] + out[2 * h + i];
    for (int i = 0; i < 2 * h - 1; ++i) out[h + i] += mid[i];
}

void orc_negacyclic_karatsuba(const uint32_t *a, const uint32_t *b, uint32_t *c, int N)
{
    uint32_t *lin = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(2 * N + 8 * N));
    uint32_t *tmp = lin + 2 * N;
    linear_karatsuba(a, b, lin, N, tmp);
    fold_negacyclic(lin, c, N);
    free(lin);
}

/* which product the gate code uses: 0 = Karatsuba (default), 1 = schoolbook, 2 = definition */
static int g_product_method = 0;
void orc_set_product_method(int m) { g_product_method = m; }

static void negacyclic_mul(const uint32_t *a, const uint32_t *b, uint32_t *c, int N)
{
    if (g_product_method == 1)      orc_negacyclic_schoolbook(a, b, c, N);
    else if (g_product_method == 2) orc_negacyclic_definition(a, b, c, N);
    else                            orc_negacyclic_karatsuba(a, b, c, N);
}

/* Multiply by the monomial X^a, 0 <= a < 2N: a signed rotation. */
void orc_mul_by_xpow(const uint32_t *p, int a, uint32_t *out, int N)
{
    for (int j = 0; j < N; ++j) {
        int e = j + a;                 /* X^j * X^a = X^e, reduce with X^N = -1 */
        int wraps = e / N;             /* 0, 1 or 2 */
        uint32_t v = p[j];
        if (wraps & 1) v = (uint32_t)0 - v;
        out[e % N] = v;
    }
}

/* ------------------------------------------------------------------ */
/* Keys                                                                */
/* ------------------------------------------------------------------ */
static size_t bk_words(const orc_params *P) { return (size_t)P->n * 2 * P->bk_l * 2 * P->N; }
static size_t ksk_rows(const orc_params *P) { return (size_t)P->N * P->ks_t * ((1u << P->ks_basebit) - 1); }

size_t orc_bk_words(const orc_params *P)  { return bk_words(P); }
size_t orc_ksk_words(const orc_params *P) { return ksk_rows(P) * (size_t)(P->n + 1); }

int orc_check_params(const orc_params *P)
{
    if (!P) return -1;
    if (P->k != 1) return -2;
    if (P->n < 1 || P->N < 2 || (P->N & (P->N - 1))) return -2;
    if (P->bk_l < 1 || P->bk_Bgbit < 1 || P->bk_l * P->bk_Bgbit > 31) return -2;
    if (P->ks_t < 1 || P->ks_basebit < 1 || P->ks_t * P->ks_basebit > 31) return -2;
    return 0;
}

/*
 * Secret keys are uniform bits (top bit of a stream word).  The bootstrapping
 * key holds, for each LWE key bit s_i, a TRGSW encryption of s_i under the ring
 * key S: 2l rows; row r = u*l + j is a fresh TRLWE encryption of zero
 * (A uniform, B = A*S + E) plus s_i * 2^(32 - Bgbit*(j+1)) on coefficient 0 of
 * component u (u = 0: the mask A, u = 1: the body B).
 * Layout: bk[i][r][c][N], c = 0 mask, c = 1 body.
 * The key-switching key holds, for each ring-key bit S_i, digit position j and
 * digit value v in 1..base-1, an LWE encryption under s of
 * v * S_i * 2^(32 - basebit*(j+1)).  Layout: ksk[i][j][v-1][n+1] (mask, then body).
 */
int orc_keygen(const orc_params *P, uint64_t seed, uint32_t *lwe_sk, uint32_t *trlwe_sk,
               uint32_t *bk, uint32_t *ksk)
{
    if (orc_check_params(P)) return -2;
    const int n = P->n, N = P->N, l = P->bk_l;
    for (int j = 0; j < n; ++j) lwe_sk[j]   = (uint32_t)(orc_rand(seed, D_LWE_SK, j) >> 63);
    for (int j = 0; j < N; ++j) trlwe_sk[j] = (uint32_t)(orc_rand(seed, D_TRLWE_SK, j) >> 63);

    if (bk) {
        for (int i = 0; i < n; ++i)
            for (int r = 0; r < 2 * l; ++r) {
                uint64_t row = (uint64_t)i * 2 * l + r;
                uint32_t *A = bk + (row * 2 + 0) * N;
                uint32_t *B = bk + (row * 2 + 1) * N;
                for (int m = 0; m < N; ++m) A[m] = rand_u32(seed, D_BK_A, row * N + m);
                negacyclic_mul(A, trlwe_sk, B, N);
                for (int m = 0; m < N; ++m)
                    B[m] += (uint32_t)orc_noise(seed, D_BK_E, row * N + m, P->bk_noise_log2);
                int u = r / l, j = r % l;
                uint32_t g = lwe_sk[i] << (32 - P->bk_Bgbit * (j + 1));
                if (u == 0) A[0] += g; else B[0] += g;
            }
    }
    if (ksk) {
        const int t = P->ks_t, bb = P->ks_basebit, base = 1 << bb;
        for (int i = 0; i < N; ++i)
            for (int j = 0; j < t; ++j)
                for (int v = 1; v < base; ++v) {
                    uint64_t q = ((uint64_t)i * t + j) * (base - 1) + (v - 1);
                    uint32_t *row = ksk + q * (size_t)(n + 1);
                    uint32_t b = 0;
                    for (int m = 0; m < n; ++m) {
                        row[m] = rand_u32(seed, D_KSK_A, q * n + m);
                        b += row[m] * lwe_sk[m];
                    }
                    b += ((uint32_t)v * trlwe_sk[i]) << (32 - bb * (j + 1));
                    b += (uint32_t)orc_noise(seed, D_KSK_E, q, P->lwe_noise_log2);
                    row[n] = b;
                }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* LWE encryption of bits: bit 1 -> +1/8, bit 0 -> -1/8 on the torus     */
/* ------------------------------------------------------------------ */
#define MU ((uint32_t)1 << 29)

void orc_encrypt(const orc_params *P, const uint32_t *lwe_sk, uint64_t seed,
                 const uint8_t *bits, size_t nbits, uint32_t *ct)
{
    const int n = P->n;
    for (size_t k = 0; k < nbits; ++k) {
        uint32_t *c = ct + k * (size_t)(n + 1);
        uint32_t b = 0;
        for (int j = 0; j < n; ++j) {
            c[j] = rand_u32(seed, D_ENC_A, k * (uint64_t)n + j);
            b += c[j] * lwe_sk[j];
        }
        b += bits[k] ? MU : (uint32_t)0 - MU;
        b += (uint32_t)orc_noise(seed, D_ENC_E, k, P->lwe_noise_log2);
        c[n] = b;
    }
}

/* phase = b - <a, s> */
uint32_t orc_phase(const uint32_t *ct, const uint32_t *sk, int n)
{
    uint32_t ph = ct[n];
    for (int j = 0; j < n; ++j) ph -= ct[j] * sk[j];
    return ph;
}

void orc_decrypt(const orc_params *P, const uint32_t *lwe_sk, const uint32_t *ct, size_t nbits,
                 uint8_t *bits)
{
    for (size_t k = 0; k < nbits; ++k)
        bits[k] = (int32_t)orc_phase(ct + k * (size_t)(P->n + 1), lwe_sk, P->n) > 0;
}

void orc_trivial(const orc_params *P, int bit, uint32_t *ct)
{
    memset(ct, 0, sizeof(uint32_t) * (size_t)(P->n + 1));
    ct[P->n] = bit ? MU : (uint32_t)0 - MU;
}

/* ------------------------------------------------------------------ */
/* One bootstrapped gate, step by step                                  */
/* ------------------------------------------------------------------ */
enum { OP_NAND = 0, OP_AND = 1, OP_OR = 2, OP_NOR = 3, OP_XOR = 4, OP_XNOR = 5 };

/*
 * Step 1: c = (0, kappa) + m * (sigma0*c0 + sigma1*c1), sigma = -1 when the
 * input is taken negated (NOT of a ciphertext is its negation, no bootstrap).
 */
int orc_gate_precombine(const orc_params *P, int op, const uint32_t *c0, int neg0,
                        const uint32_t *c1, int neg1, uint32_t *c)
{
    uint32_t kappa; uint32_t m;
    switch (op) {
    case OP_NAND: kappa = MU;               m = (uint32_t)-1; break;
    case OP_AND:  kappa = (uint32_t)0 - MU; m = 1;            break;
    case OP_OR:   kappa = MU;               m = 1;            break;
    case OP_NOR:  kappa = (uint32_t)0 - MU; m = (uint32_t)-1; break;
    case OP_XOR:  kappa = 2 * MU;           m = 2;            break;
    case OP_XNOR: kappa = (uint32_t)0 - 2 * MU; m = (uint32_t)-2; break;
    default: return -2;
    }
    for (int j = 0; j <= P->n; ++j) {
        uint32_t x0 = neg0 ? (uint32_t)0 - c0[j] : c0[j];
        uint32_t x1 = neg1 ? (uint32_t)0 - c1[j] : c1[j];
        c[j] = m * (x0 + x1);
    }
    c[P->n] += kappa;
    return 0;
}

static int ilog2(int x) { int r = 0; while ((1 << r) < x) ++r; return r; }

/* Step 2: round each torus word to the nearest multiple of 1/2N (half up). */
void orc_modswitch(const orc_params *P, const uint32_t *c, uint32_t *bar)
{
    int sh = 32 - (ilog2(P->N) + 1);
    for (int j = 0; j <= P->n; ++j)
        bar[j] = ((c[j] + ((uint32_t)1 << (sh - 1))) >> sh) & (uint32_t)(2 * P->N - 1);
}

/* Step 3: ACC = (0, X^{-bbar} * v), v = 1/8 on every coefficient.  acc[0..N) mask, acc[N..2N) body. */
void orc_acc_init(const orc_params *P, uint32_t bbar, uint32_t *acc)
{
    const int N = P->N;
    uint32_t *v = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N);
    for (int j = 0; j < N; ++j) { acc[j] = 0; v[j] = MU; }
    orc_mul_by_xpow(v, (int)((2 * N - bbar) % (2 * N)), acc + N, N);
    free(v);
}

/*
 * Gadget decomposition of one torus word into l signed digits in
 * [-Bg/2, Bg/2), nearest-multiple rounding at the last digit:
 *   x ~ sum_j d_j * 2^(32 - Bgbit*(j+1)),  residue in [-2^(31-l*Bgbit), 2^(31-l*Bgbit)).
 */
void orc_decompose(const orc_params *P, uint32_t x, int32_t *d)
{
    const int l = P->bk_l, bg = P->bk_Bgbit;
    uint32_t offset = (uint32_t)1 << (32 - l * bg - 1);
    for (int j = 0; j < l; ++j) offset += ((uint32_t)1 << (bg - 1)) << (32 - bg * (j + 1));
    uint32_t xp = x + offset;
    for (int j = 0; j < l; ++j)
        d[j] = (int32_t)((xp >> (32 - bg * (j + 1))) & (((uint32_t)1 << bg) - 1)) - (1 << (bg - 1));
}

/*
 * External product: out = BK_i [.] (D_A, D_B)
 *   = sum_{u in {A,B}} sum_j dec_j(D_u) * row(u, j)      (a TRLWE sample)
 * bk_i points at bk[i]; D and out are 2N words (mask, body).
 */
void orc_external_product(const orc_params *P, const uint32_t *bk_i, const uint32_t *D, uint32_t *out)
{
    const int N = P->N, l = P->bk_l;
    uint32_t *digit = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N * 2);
    uint32_t *prod = digit + N;
    int32_t d[32];
    memset(out, 0, sizeof(uint32_t) * 2 * (size_t)N);
    for (int u = 0; u < 2; ++u)
        for (int j = 0; j < l; ++j) {
            for (int m = 0; m < N; ++m) { orc_decompose(P, D[u * N + m], d); digit[m] = (uint32_t)d[j]; }
            const uint32_t *row = bk_i + (size_t)(u * l + j) * 2 * N;
            for (int c = 0; c < 2; ++c) {
                negacyclic_mul(digit, row + c * N, prod, N);
                for (int m = 0; m < N; ++m) out[c * N + m] += prod[m];
            }
        }
    free(digit);
}

/* Step 4: for i = 0..n-1 in order:  ACC += BK_i [.] (X^{abar_i} * ACC - ACC). */
void orc_blind_rotate(const orc_params *P, const uint32_t *bk, const uint32_t *bar, uint32_t *acc)
{
    const int N = P->N;
    uint32_t *D = (uint32_t *)malloc(sizeof(uint32_t) * 4 * (size_t)N);
    uint32_t *E = D + 2 * N;
    for (int i = 0; i < P->n; ++i) {
        if (bar[i] == 0) continue;                    /* D would be identically zero */
        for (int c = 0; c < 2; ++c) {
            orc_mul_by_xpow(acc + c * N, (int)bar[i], D + c * N, N);
            for (int m = 0; m < N; ++m) D[c * N + m] -= acc[c * N + m];
        }
        orc_external_product(P, bk + (size_t)i * 2 * P->bk_l * 2 * N, D, E);
        for (int m = 0; m < 2 * N; ++m) acc[m] += E[m];
    }
    free(D);
}

/* Step 5: the constant coefficient of the TRLWE phase, as an LWE sample under the N ring-key bits. */
void orc_sample_extract(const orc_params *P, const uint32_t *acc, uint32_t *ext)
{
    const int N = P->N;
    ext[0] = acc[0];
    for (int j = 1; j < N; ++j) ext[j] = (uint32_t)0 - acc[N - j];
    ext[N] = acc[N];
}

/* Step 6: key switch to the n-bit key with base-2^basebit digits of the rounded mask words. */
void orc_key_switch(const orc_params *P, const uint32_t *ksk, const uint32_t *ext, uint32_t *out)
{
    const int n = P->n, N = P->N, t = P->ks_t, bb = P->ks_basebit, base = 1 << bb;
    for (int m = 0; m < n; ++m) out[m] = 0;
    out[n] = ext[N];
    uint32_t round = (uint32_t)1 << (32 - t * bb - 1);
    for (int i = 0; i < N; ++i) {
        uint32_t ai = ext[i] + round;
        for (int j = 0; j < t; ++j) {
            uint32_t v = (ai >> (32 - bb * (j + 1))) & (uint32_t)(base - 1);
            if (v == 0) continue;
            const uint32_t *row = ksk + (((size_t)i * t + j) * (base - 1) + (v - 1)) * (size_t)(n + 1);
            for (int m = 0; m <= n; ++m) out[m] -= row[m];
        }
    }
}

/* The whole gate. */
int orc_gate(const orc_params *P, const uint32_t *bk, const uint32_t *ksk, int op,
             const uint32_t *c0, int neg0, const uint32_t *c1, int neg1, uint32_t *out)
{
    const int n = P->n, N = P->N;
    uint32_t *c = (uint32_t *)malloc(sizeof(uint32_t) * ((size_t)2 * (n + 1) + 2 * N + N + 1));
    uint32_t *bar = c + (n + 1), *acc = bar + (n + 1), *ext = acc + 2 * N;
    int rc = orc_gate_precombine(P, op, c0, neg0, c1, neg1, c);
    if (rc == 0) {
        orc_modswitch(P, c, bar);
        orc_acc_init(P, bar[n], acc);
        orc_blind_rotate(P, bk, bar, acc);
        orc_sample_extract(P, acc, ext);
        orc_key_switch(P, ksk, ext, out);
    }
    free(c);
    return rc;
}

/*
 * Steps 2-5 on an already pre-combined sample: the bootstrapped value as an LWE sample under the
 * ring key (N+1 words), not yet key-switched.
 */
void orc_bootstrap_extract(const orc_params *P, const uint32_t *bk, const uint32_t *c, uint32_t *ext)
{
    const int n = P->n, N = P->N;
    uint32_t *bar = (uint32_t *)malloc(sizeof(uint32_t) * ((size_t)(n + 1) + 2 * N));
    uint32_t *acc = bar + (n + 1);
    orc_modswitch(P, c, bar);
    orc_acc_init(P, bar[n], acc);
    orc_blind_rotate(P, bk, bar, acc);
    orc_sample_extract(P, acc, ext);
    free(bar);
}

/*
 * Multiplexer MUX(s, a, b) = s ? a : b, the three-input gate of Algorithm 1 (TAPAS Sec. 4.1;
 * "MUX(s, a, b) returns a if s = 1 and b otherwise").  CGGI evaluates it with two blind
 * rotations and one key switch: u1 = bootstrap(AND(s, a)), u2 = bootstrap(AND(NOT s, b)), both
 * left under the ring key; exactly one or none of them is true, so u1 + u2 + 1/8 is +-1/8 and
 * is key-switched once.  neg flags take an input negated, as for the two-input gates.
 */
int orc_mux(const orc_params *P, const uint32_t *bk, const uint32_t *ksk,
            const uint32_t *s, int negs, const uint32_t *a, int nega, const uint32_t *b, int negb,
            uint32_t *out)
{
    const int n = P->n, N = P->N;
    uint32_t *c = (uint32_t *)malloc(sizeof(uint32_t) * ((size_t)(n + 1) + 2 * (N + 1)));
    uint32_t *u1 = c + (n + 1), *u2 = u1 + (N + 1);
    orc_gate_precombine(P, OP_AND, s, negs, a, nega, c);
    orc_bootstrap_extract(P, bk, c, u1);
    orc_gate_precombine(P, OP_AND, s, !negs, b, negb, c);
    orc_bootstrap_extract(P, bk, c, u2);
    for (int j = 0; j <= N; ++j) u1[j] += u2[j];
    u1[N] += MU;
    orc_key_switch(P, ksk, u1, out);
    free(c);
    return 0;
}

/* gate record shared by the batch entry point: 16 bytes */
typedef struct { uint8_t op, neg0, neg1, pad; int32_t in0, in1, out; } orc_gate_rec;

/*
 * Evaluate `count` mutually independent gates over a wire array
 * (wires[w] is an LWE sample of n+1 words).  Gates are independent, so the
 * loop may run on several threads; each gate is still the plain orc_gate.
 * A multiplexer is two consecutive records with the same selector and output:
 * {OP_MUX, negs, nega, s, a, out} then {OP_MUX_ELSE, negs, negb, s, b, out}.
 */
enum { OP_MUX = 6, OP_MUX_ELSE = 7 };

int orc_gate_batch(const orc_params *P, const uint32_t *bk, const uint32_t *ksk,
                   const orc_gate_rec *g, size_t count, uint32_t *wires, int threads)
{
    int bad = 0;
    const size_t w = (size_t)P->n + 1;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (long i = 0; i < (long)count; ++i) {
        int rc = 0;
        if (g[i].op == OP_MUX_ELSE) {
            if (i == 0 || g[i - 1].op != OP_MUX) rc = -2;      /* evaluated with its first half */
        } else if (g[i].op == OP_MUX) {
            if (i + 1 >= (long)count || g[i + 1].op != OP_MUX_ELSE || g[i + 1].in0 != g[i].in0 ||
                g[i + 1].out != g[i].out || g[i + 1].neg0 != g[i].neg0)
                rc = -2;
            else
                rc = orc_mux(P, bk, ksk, wires + g[i].in0 * w, g[i].neg0, wires + g[i].in1 * w, g[i].neg1,
                             wires + g[i + 1].in1 * w, g[i + 1].neg1, wires + g[i].out * w);
        } else {
            rc = orc_gate(P, bk, ksk, g[i].op, wires + g[i].in0 * w, g[i].neg0,
                          wires + g[i].in1 * w, g[i].neg1, wires + g[i].out * w);
        }
        if (rc) {
#pragma omp atomic write
            bad = 1;
        }
    }
    return bad ? -2 : 0;
}
