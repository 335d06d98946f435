// Sanitizer run of the library's host code (AddressSanitizer + UndefinedBehaviorSanitizer):
// key generation, export / import, encryption, decryption, every lowering (threaded and not)
// and the argument checks, at a toy parameter set.  The device kernels are not part of this
// build: their launchers are stubs that must never be reached, because no GPU call can succeed
// here.  Built and run by tests/test_sanitizers.py.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../paper_1806_03461_amd/csrc/kernels.h"

namespace tfhe {
static int unreachable(const char *what) { std::fprintf(stderr, "device launcher %s reached\n", what); std::abort(); }
size_t blind_rotate_lds_bytes(int) { return 0; }
int launch_bk_to_spectrum(const uint32_t *, double2 *, const double2 *, int, hipStream_t) { return unreachable("bk"); }
int launch_blind_rotate(const BlindRotateArgs &, hipStream_t) { return unreachable("blind_rotate"); }
int launch_key_switch(const KeySwitchArgs &, hipStream_t) { return unreachable("key_switch"); }
size_t ksk_tiles_bytes() { return 0; }
int launch_ksk_to_tiles(const uint32_t *, int, int, void *, hipStream_t) { return unreachable("tiles"); }
int launch_mux_combine(uint32_t *, const tfhe_gate_rec *, size_t, hipStream_t) { return unreachable("mux"); }
int launch_gather_outputs(const uint32_t *, const tfhe_out_ref *, uint32_t *, size_t, int, hipStream_t) { return unreachable("gather"); }
int launch_fill_trivial(uint32_t *, int, int, hipStream_t) { return unreachable("fill"); }
int prepare_kernels() { return unreachable("prepare"); }
int measure_fp64_fma_peak(hipStream_t, double *, double *) { return unreachable("peak"); }
uint32_t *static_scratch_ptr() { return nullptr; }
size_t static_scratch_gates() { return 4096; }
}  // namespace tfhe

#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #cond); return 1; } } while (0)

int main() {
    tfhe_params P{16, 32, 1, 2, 10, 8, 2, -15, -25};
    tfhe_secret_key *sk = nullptr;
    tfhe_cloud_key *ck = nullptr;
    CHECK(tfhe_keygen(&P, 4242, &sk, &ck) == TFHE_OK);

    // export, import, export again
    std::vector<std::vector<uint32_t>> parts(4);
    for (int which = 0; which < 4; ++which) {
        size_t len = 0;
        const void *key = which < 2 ? (const void *)sk : (const void *)ck;
        CHECK(tfhe_export_key(key, which, nullptr, &len) == TFHE_OK);
        parts[which].resize(len / 4);
        CHECK(tfhe_export_key(key, which, parts[which].data(), &len) == TFHE_OK);
        size_t small_len = len - 4;
        CHECK(tfhe_export_key(key, which, parts[which].data(), &small_len) == TFHE_E_SIZE);
    }
    tfhe_secret_key *sk2 = nullptr;
    tfhe_cloud_key *ck2 = nullptr;
    CHECK(tfhe_import_keys(&P, parts[0].data(), parts[1].data(), parts[2].data(), parts[3].data(), &sk2, &ck2) == TFHE_OK);
    CHECK(tfhe_import_keys(&P, nullptr, parts[1].data(), parts[2].data(), parts[3].data(), &sk2, nullptr) == TFHE_E_NULL);

    // encrypt with one key object, decrypt with the other
    const uint8_t bits[5] = {1, 0, 0, 1, 1};
    uint8_t back[5];
    std::vector<uint32_t> ct(5 * (P.n + 1));
    CHECK(tfhe_encrypt(sk, 7, bits, 5, ct.data()) == TFHE_OK);
    CHECK(tfhe_decrypt(sk2, ct.data(), 5, back) == TFHE_OK);
    CHECK(std::memcmp(bits, back, 5) == 0);
    CHECK(tfhe_encrypt(sk, 7, bits, 0, ct.data()) == TFHE_OK);

    // lowerings: every flag combination that is allowed, serial and threaded
    const int d = 23, p = 9;
    std::vector<int8_t> W((size_t)d * p);
    std::vector<int32_t> T(p);
    for (size_t i = 0; i < W.size(); ++i) W[i] = (int8_t)((i * 7 + i / 5) % 3 - 1);
    for (int j = 0; j < p; ++j) T[j] = 3 + j;
    const uint32_t flags[] = {0, TFHE_LOWER_MUX_COMPARATOR, TFHE_LOWER_PLUS_ONE, TFHE_LOWER_SHARE_GATES,
                              TFHE_LOWER_PLUS_ONE | TFHE_LOWER_SHARE_GATES, TFHE_LOWER_SORTING_NETWORK};
    for (const char *threads : {"1", "3"}) {
        setenv("TFHE_LOWER_THREADS", threads, 1);
        for (uint32_t f : flags) {
            tfhe_gate_rec *g = nullptr; tfhe_out_ref *o = nullptr; size_t ng = 0, no = 0, nw = 0;
            CHECK(bnn_dense_lower_opts(d, W.data(), T.data(), p, 0, f, &g, &ng, &o, &no, &nw) == TFHE_OK);
            CHECK(no == (size_t)p && nw >= (size_t)d + 2);
            {   // the wire-pool schedule of the layer calls on the same circuit
                tfhe_gate_rec *planned = nullptr; size_t pool = 0, depths = 0;
                CHECK(tfhe_plan_wire_pool(g, ng, nw, (size_t)d + 2, o, no, &planned, &pool, &depths) == TFHE_OK);
                CHECK(pool >= (size_t)d + 2 && pool <= nw && depths >= 1);
                for (size_t k = 0; k < ng; ++k)
                    CHECK((size_t)planned[k].in0 < pool && (size_t)planned[k].in1 < pool && (size_t)planned[k].out < pool);
                tfhe_free_buffer(planned);
                tfhe_gate_rec cyclic = g[0];
                cyclic.in0 = cyclic.out;
                CHECK(tfhe_plan_wire_pool(&cyclic, 1, nw, (size_t)d + 2, nullptr, 0, &planned, &pool, &depths) == TFHE_E_PARAM);
            }
            tfhe_free_buffer(g); tfhe_free_buffer(o);
            if (f & TFHE_LOWER_MUX_COMPARATOR) continue;
            std::vector<int8_t> K(3 * 2 * 3 * 3);
            for (size_t i = 0; i < K.size(); ++i) K[i] = (int8_t)(i % 2 ? 1 : -1);
            const int32_t Tc[3] = {8, 9, 10};
            CHECK(bnn_conv_lower_opts(2, 5, 4, K.data(), 3, 3, 3, 1, 1, Tc, f, &g, &ng, &o, &no, &nw) == TFHE_OK);
            CHECK(no == (size_t)3 * 5 * 4);
            tfhe_free_buffer(g); tfhe_free_buffer(o);
        }
        tfhe_gate_rec *g = nullptr; tfhe_out_ref *o = nullptr; size_t ng = 0, no = 0, nw = 0;
        CHECK(bnn_dense_lower(d, W.data(), nullptr, p, 6, &g, &ng, &o, &no, &nw) == TFHE_OK);
        CHECK(no == (size_t)p * 6);
        tfhe_free_buffer(g); tfhe_free_buffer(o);
    }
    // refused arguments leave nothing behind
    {
        tfhe_gate_rec *g = nullptr; tfhe_out_ref *o = nullptr; size_t ng = 0, no = 0, nw = 0;
        W[3] = 2;
        CHECK(bnn_dense_lower(d, W.data(), T.data(), p, 0, &g, &ng, &o, &no, &nw) == TFHE_E_PARAM);
        CHECK(bnn_dense_lower(0, W.data(), T.data(), p, 0, &g, &ng, &o, &no, &nw) == TFHE_E_SIZE);
        CHECK(bnn_dense_lower_opts(d, W.data(), T.data(), p, 0, 64, &g, &ng, &o, &no, &nw) == TFHE_E_PARAM);
        tfhe_params bad = P;
        bad.N = 48;
        tfhe_secret_key *s3 = nullptr;
        CHECK(tfhe_keygen(&bad, 1, &s3, nullptr) == TFHE_E_PARAM && s3 == nullptr);
        CHECK(std::strlen(tfhe_last_error()) > 0);
    }
    tfhe_free_secret_key(sk); tfhe_free_secret_key(sk2);
    tfhe_free_cloud_key(ck); tfhe_free_cloud_key(ck2);
    std::puts("host-code sanitizer run: ok");
    return 0;
}
