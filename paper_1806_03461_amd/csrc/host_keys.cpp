// Client-side host code: deterministic key generation, encryption, decryption, key export.
//
// The TAPAS paper (Sec. 2) has the client generate keys and encrypt its bits; it does not
// describe the scheme (it cites CGGI, Sec. 3.1.2).  The construction here is the public
// one: binary LWE / ring keys, a TRGSW bootstrapping key with a power-of-two gadget and an
// LWE key-switching key with one row per non-zero digit value.  Randomness is a
// counter-addressed SplitMix64 stream per purpose, so that any element can be produced
// independently and in any order; the noise is an integer-only sum of twelve uniform words.
#include <cstring>
#include <new>

#include "common.h"

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

inline uint64_t finalize(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

// A random-access view of one SplitMix64 sequence: element i is output i+1 of the
// generator whose state starts at `origin`.
class Stream {
public:
    enum Purpose : uint32_t { kLweKey = 1, kRingKey = 2, kBkMask = 3, kBkNoise = 4,
                              kKsMask = 5, kKsNoise = 6, kEncMask = 7, kEncNoise = 8 };
    Stream(uint64_t seed, Purpose purpose) : origin_(finalize(seed + kGolden * purpose)) {}
    uint64_t word64(uint64_t i) const { return finalize(origin_ + kGolden * (i + 1)); }
    uint32_t word32(uint64_t i) const { return (uint32_t)(word64(i) >> 32); }
    uint32_t bit(uint64_t i) const { return (uint32_t)(word64(i) >> 63); }
    // Sample i of a centred bell-shaped integer with standard deviation 2^(32 + log2sd):
    // twelve uniform 32-bit words summed, mean removed, divided by 2^-log2sd rounding half up.
    uint32_t noise(uint64_t i, int log2sd) const {
        const int shift = -log2sd;
        if (shift < 1 || shift >= 40) return 0;
        int64_t sum = -((int64_t)6 << 32);
        for (uint64_t j = 0; j < 12; ++j) sum += word32(12 * i + j);
        const int64_t biased = sum + ((int64_t)1 << (shift - 1));
        const int64_t q = biased >= 0 ? (biased >> shift)
                                      : -((-biased + (((int64_t)1 << shift) - 1)) >> shift);
        return (uint32_t)q;
    }
private:
    uint64_t origin_;
};

// body += mask * key in Z_{2^32}[X]/(X^N+1) for a 0/1 key polynomial: each set key bit j
// contributes the mask shifted by j places, the part that wraps past X^N negated.
void add_mask_times_binary_key(const uint32_t *mask, const uint32_t *key, uint32_t *body, int N) {
    for (int j = 0; j < N; ++j) {
        if (!key[j]) continue;
        for (int m = 0; m < N - j; ++m) body[m + j] += mask[m];
        for (int m = N - j; m < N; ++m) body[m + j - N] -= mask[m];
    }
}

constexpr uint32_t kEighth = 1u << 29;

}  // namespace

namespace tfhe {

static thread_local char g_error[512] = "";

int set_error(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return code;
}

int check_params_host(const tfhe_params *p) {
    if (!p) return set_error(TFHE_E_NULL, "params is NULL");
    if (p->k != 1) return set_error(TFHE_E_PARAM, "k must be 1 (got %d)", p->k);
    if (p->n < 1 || p->n > (1 << 16)) return set_error(TFHE_E_PARAM, "n out of range (%d)", p->n);
    if (p->N < 2 || p->N > (1 << 14) || (p->N & (p->N - 1)))
        return set_error(TFHE_E_PARAM, "N must be a power of two in [2, 16384] (got %d)", p->N);
    if (p->bk_l < 1 || p->bk_Bgbit < 1 || p->bk_l * p->bk_Bgbit > 31)
        return set_error(TFHE_E_PARAM, "bad gadget (l=%d, Bgbit=%d)", p->bk_l, p->bk_Bgbit);
    if (p->ks_t < 1 || p->ks_basebit < 1 || p->ks_t * p->ks_basebit > 31)
        return set_error(TFHE_E_PARAM, "bad key-switch digits (t=%d, basebit=%d)", p->ks_t, p->ks_basebit);
    if (p->lwe_noise_log2 >= 0 || p->bk_noise_log2 >= 0)
        return set_error(TFHE_E_PARAM, "noise_log2 must be negative");
    return TFHE_OK;
}

int check_params_gpu(const tfhe_params *p) {
    int rc = check_params_host(p);
    if (rc) return rc;
    if (p->N != 1024 || p->bk_l != 2 || p->bk_Bgbit > 10 || p->n > 1024 ||
        p->ks_t * p->ks_basebit > 24 || p->ks_basebit > 4)
        return set_error(TFHE_E_PARAM,
                         "GPU path needs N=1024, l=2, Bgbit<=10, n<=1024, t*basebit<=24, basebit<=4");
    return TFHE_OK;
}

}  // namespace tfhe

using tfhe::set_error;

extern "C" {

const char *tfhe_last_error(void) { return tfhe::g_error; }

void tfhe_default_params(tfhe_params *p) {
    if (!p) return;
    *p = tfhe_params{500, 1024, 1, 2, 10, 8, 2, -15, -25};
}

int tfhe_keygen(const tfhe_params *p, uint64_t seed, tfhe_secret_key **sk_out, tfhe_cloud_key **ck_out) {
    if (int rc = tfhe::check_params_host(p)) return rc;
    if (!sk_out && !ck_out) return set_error(TFHE_E_NULL, "both output pointers are NULL");
    const int n = p->n, N = p->N, l = p->bk_l;

    tfhe_secret_key *sk = new (std::nothrow) tfhe_secret_key();
    if (!sk) return set_error(TFHE_E_ALLOC, "out of memory");
    sk->magic = TFHE_SK_MAGIC;
    sk->params = *p;
    sk->lwe.resize(n);
    sk->trlwe.resize(N);
    {
        Stream a(seed, Stream::kLweKey), b(seed, Stream::kRingKey);
        for (int j = 0; j < n; ++j) sk->lwe[j] = a.bit(j);
        for (int j = 0; j < N; ++j) sk->trlwe[j] = b.bit(j);
    }

    if (ck_out) {
        tfhe_cloud_key *ck = new (std::nothrow) tfhe_cloud_key();
        if (!ck) { delete sk; return set_error(TFHE_E_ALLOC, "out of memory"); }
        ck->magic = TFHE_CK_MAGIC;
        ck->params = *p;
        try {
            ck->bk_raw.assign((size_t)n * tfhe::bk_row_words(*p), 0);
            ck->ksk_raw.assign(tfhe::ksk_rows(*p) * (size_t)(n + 1), 0);
        } catch (const std::bad_alloc &) {
            delete ck; delete sk;
            return set_error(TFHE_E_ALLOC, "out of memory for the cloud key");
        }
        // Bootstrapping key: TRGSW(s_i) = 2l fresh TRLWE encryptions of zero plus s_i times
        // the gadget: row (u, j) gets s_i * 2^(32 - Bgbit (j+1)) on X^0 of component u.
        Stream mask(seed, Stream::kBkMask), err(seed, Stream::kBkNoise);
        for (int i = 0; i < n; ++i) {
            for (int r = 0; r < 2 * l; ++r) {
                const uint64_t sample = (uint64_t)i * 2 * l + r;
                uint32_t *A = &ck->bk_raw[(sample * 2) * N];
                uint32_t *B = A + N;
                for (int m = 0; m < N; ++m) {
                    A[m] = mask.word32(sample * N + m);
                    B[m] = err.noise(sample * N + m, p->bk_noise_log2);
                }
                add_mask_times_binary_key(A, sk->trlwe.data(), B, N);
                const uint32_t gadget = sk->lwe[i] << (32 - p->bk_Bgbit * (r % l + 1));
                (r < l ? A : B)[0] += gadget;
            }
        }
        // Key-switching key: row (i, j, v) encrypts v * S_i * 2^(32 - basebit (j+1)) under s.
        Stream kmask(seed, Stream::kKsMask), kerr(seed, Stream::kKsNoise);
        const int values = (1 << p->ks_basebit) - 1;
        const uint64_t rows = tfhe::ksk_rows(*p);
        for (uint64_t q = 0; q < rows; ++q) {
            const int v = (int)(q % values) + 1;
            const int j = (int)((q / values) % p->ks_t);
            const int i = (int)(q / values / p->ks_t);
            uint32_t *row = &ck->ksk_raw[q * (size_t)(n + 1)];
            uint32_t body = kerr.noise(q, p->lwe_noise_log2);
            for (int m = 0; m < n; ++m) {
                row[m] = kmask.word32(q * n + m);
                if (sk->lwe[m]) body += row[m];
            }
            if (sk->trlwe[i]) body += (uint32_t)v << (32 - p->ks_basebit * (j + 1));
            row[n] = body;
        }
        *ck_out = ck;
    }
    if (sk_out) *sk_out = sk; else delete sk;
    return TFHE_OK;
}

static int tfhe_encrypt_impl(const tfhe_secret_key *sk, uint64_t seed, const uint8_t *bits, size_t nbits,
                 uint32_t *ct) {
    if (!sk || (nbits && (!bits || !ct))) return set_error(TFHE_E_NULL, "NULL argument to tfhe_encrypt");
    if (sk->magic != TFHE_SK_MAGIC) return set_error(TFHE_E_PARAM, "not a secret key");
    const int n = sk->params.n;
    Stream mask(seed, Stream::kEncMask), err(seed, Stream::kEncNoise);
    for (size_t s = 0; s < nbits; ++s) {
        uint32_t *c = ct + s * (size_t)(n + 1);
        uint32_t body = (bits[s] ? kEighth : 0u - kEighth) + err.noise(s, sk->params.lwe_noise_log2);
        for (int j = 0; j < n; ++j) {
            c[j] = mask.word32(s * (uint64_t)n + j);
            if (sk->lwe[j]) body += c[j];
        }
        c[n] = body;
    }
    return TFHE_OK;
}

int tfhe_encrypt(const tfhe_secret_key *sk, uint64_t seed, const uint8_t *bits, size_t nbits,
                 uint32_t *ct) {
    return tfhe::guarded([&]() -> int { return tfhe_encrypt_impl(sk, seed, bits, nbits, ct); });
}

static int tfhe_decrypt_impl(const tfhe_secret_key *sk, const uint32_t *ct, size_t nbits, uint8_t *bits) {
    if (!sk || (nbits && (!bits || !ct))) return set_error(TFHE_E_NULL, "NULL argument to tfhe_decrypt");
    if (sk->magic != TFHE_SK_MAGIC) return set_error(TFHE_E_PARAM, "not a secret key");
    const int n = sk->params.n;
    for (size_t s = 0; s < nbits; ++s) {
        const uint32_t *c = ct + s * (size_t)(n + 1);
        uint32_t phase = c[n];
        for (int j = 0; j < n; ++j)
            if (sk->lwe[j]) phase -= c[j];
        bits[s] = (int32_t)phase > 0;
    }
    return TFHE_OK;
}

int tfhe_decrypt(const tfhe_secret_key *sk, const uint32_t *ct, size_t nbits, uint8_t *bits) {
    return tfhe::guarded([&]() -> int { return tfhe_decrypt_impl(sk, ct, nbits, bits); });
}

int tfhe_trivial(const tfhe_params *p, int bit, uint32_t *ct) {
    if (!p || !ct) return set_error(TFHE_E_NULL, "NULL argument to tfhe_trivial");
    if (p->n < 1) return set_error(TFHE_E_PARAM, "bad n");
    memset(ct, 0, sizeof(uint32_t) * (size_t)p->n);
    ct[p->n] = bit ? kEighth : 0u - kEighth;
    return TFHE_OK;
}

int tfhe_get_params(const void *key, int is_cloud_key, tfhe_params *out) {
    if (!key || !out) return set_error(TFHE_E_NULL, "NULL argument to tfhe_get_params");
    if (is_cloud_key) {
        auto *ck = (const tfhe_cloud_key *)key;
        if (ck->magic != TFHE_CK_MAGIC) return set_error(TFHE_E_PARAM, "not a cloud key");
        *out = ck->params;
    } else {
        auto *sk = (const tfhe_secret_key *)key;
        if (sk->magic != TFHE_SK_MAGIC) return set_error(TFHE_E_PARAM, "not a secret key");
        *out = sk->params;
    }
    return TFHE_OK;
}

static int tfhe_export_key_impl(const void *key, int which, void *buf, size_t *len) {
    if (!key || !len) return set_error(TFHE_E_NULL, "NULL argument to tfhe_export_key");
    const std::vector<uint32_t> *src = nullptr;
    if (which == TFHE_KEY_LWE_SK || which == TFHE_KEY_TRLWE_SK) {
        auto *sk = (const tfhe_secret_key *)key;
        if (sk->magic != TFHE_SK_MAGIC) return set_error(TFHE_E_PARAM, "not a secret key");
        src = which == TFHE_KEY_LWE_SK ? &sk->lwe : &sk->trlwe;
    } else if (which == TFHE_KEY_BK_RAW || which == TFHE_KEY_KSK_RAW) {
        auto *ck = (const tfhe_cloud_key *)key;
        if (ck->magic != TFHE_CK_MAGIC) return set_error(TFHE_E_PARAM, "not a cloud key");
        src = which == TFHE_KEY_BK_RAW ? &ck->bk_raw : &ck->ksk_raw;
    } else {
        return set_error(TFHE_E_PARAM, "unknown key part %d", which);
    }
    const size_t bytes = src->size() * sizeof(uint32_t);
    if (!buf) { *len = bytes; return TFHE_OK; }
    if (*len < bytes) { *len = bytes; return set_error(TFHE_E_SIZE, "buffer too small, need %zu bytes", bytes); }
    memcpy(buf, src->data(), bytes);
    *len = bytes;
    return TFHE_OK;
}

int tfhe_export_key(const void *key, int which, void *buf, size_t *len) {
    return tfhe::guarded([&]() -> int { return tfhe_export_key_impl(key, which, buf, len); });
}

static int tfhe_import_keys_impl(const tfhe_params *p, const uint32_t *lwe_sk, const uint32_t *trlwe_sk,
                                 const uint32_t *bk_raw, const uint32_t *ksk_raw, tfhe_secret_key **sk_out,
                                 tfhe_cloud_key **ck_out) {
    if (int rc = tfhe::check_params_host(p)) return rc;
    if (!sk_out && !ck_out) return set_error(TFHE_E_NULL, "both output pointers are NULL");
    if (sk_out && (!lwe_sk || !trlwe_sk)) return set_error(TFHE_E_NULL, "a secret key needs lwe_sk and trlwe_sk");
    if (ck_out && (!bk_raw || !ksk_raw)) return set_error(TFHE_E_NULL, "a cloud key needs bk_raw and ksk_raw");
    if (sk_out) {
        for (int j = 0; j < p->n; ++j)
            if (lwe_sk[j] > 1) return set_error(TFHE_E_PARAM, "lwe_sk[%d] is not a bit", j);
        for (int j = 0; j < p->N; ++j)
            if (trlwe_sk[j] > 1) return set_error(TFHE_E_PARAM, "trlwe_sk[%d] is not a bit", j);
    }
    tfhe_secret_key *sk = nullptr;
    tfhe_cloud_key *ck = nullptr;
    struct Guard {                       // nothing is handed out unless everything succeeded
        tfhe_secret_key *&sk;
        tfhe_cloud_key *&ck;
        ~Guard() { delete sk; delete ck; }
    } guard{sk, ck};
    if (sk_out) {
        sk = new tfhe_secret_key();
        sk->magic = TFHE_SK_MAGIC;
        sk->params = *p;
        sk->lwe.assign(lwe_sk, lwe_sk + p->n);
        sk->trlwe.assign(trlwe_sk, trlwe_sk + p->N);
    }
    if (ck_out) {
        ck = new tfhe_cloud_key();
        ck->magic = TFHE_CK_MAGIC;
        ck->params = *p;
        ck->bk_raw.assign(bk_raw, bk_raw + (size_t)p->n * tfhe::bk_row_words(*p));
        ck->ksk_raw.assign(ksk_raw, ksk_raw + tfhe::ksk_rows(*p) * (size_t)(p->n + 1));
    }
    if (sk_out) *sk_out = sk;
    if (ck_out) *ck_out = ck;
    sk = nullptr; ck = nullptr;
    return TFHE_OK;
}

int tfhe_import_keys(const tfhe_params *p, const uint32_t *lwe_sk, const uint32_t *trlwe_sk,
                     const uint32_t *bk_raw, const uint32_t *ksk_raw, tfhe_secret_key **sk,
                     tfhe_cloud_key **ck) {
    return tfhe::guarded(
        [&]() -> int { return tfhe_import_keys_impl(p, lwe_sk, trlwe_sk, bk_raw, ksk_raw, sk, ck); });
}

void tfhe_free_secret_key(tfhe_secret_key *sk) {
    if (sk && sk->magic == TFHE_SK_MAGIC) { sk->magic = 0; delete sk; }
}

void tfhe_free_buffer(void *p) { free(p); }

}  // extern "C"
