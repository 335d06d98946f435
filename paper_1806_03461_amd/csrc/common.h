// Internal declarations shared by the host-side sources of the library.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <exception>
#include <new>
#include <vector>

#include <hip/hip_runtime.h>

#include "../../include/tfhe_mi355x.h"

namespace tfhe {

int set_error(int code, const char *fmt, ...);

#define TFHE_HIP(call)                                                                      \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return tfhe::set_error(TFHE_E_HIP, "%s failed: %s (%s:%d)", #call,              \
                                   hipGetErrorString(e_), __FILE__, __LINE__);              \
    } while (0)

// thrown by the lowering when wire numbers would leave int32
struct CircuitTooLarge {};

// Runs an entry point's body: no C++ exception leaves the C ABI.
template <class F>
int guarded(F &&body) {
    try {
        return body();
    } catch (const CircuitTooLarge &) {
        return set_error(TFHE_E_SIZE, "the circuit needs more than 2^31 - 1 wires");
    } catch (const std::bad_alloc &) {
        return set_error(TFHE_E_ALLOC, "out of host memory");
    } catch (const std::exception &e) {
        return set_error(TFHE_E_ALLOC, "unexpected failure: %s", e.what());
    } catch (...) {
        return set_error(TFHE_E_ALLOC, "unexpected failure");
    }
}

int check_params_host(const tfhe_params *p);   // what keygen / encrypt accept
int check_params_gpu(const tfhe_params *p);    // what the kernels accept

inline size_t bk_row_words(const tfhe_params &p) { return (size_t)2 * p.bk_l * 2 * p.N; }
inline size_t ksk_rows(const tfhe_params &p) {
    return (size_t)p.N * p.ks_t * ((1u << p.ks_basebit) - 1);
}

// A grow-only device buffer.
struct DeviceBuffer {
    void *ptr = nullptr;
    size_t bytes = 0;
    int reserve(size_t want);
    void release();
};

// A grow-only pinned host buffer for uploads that must not block: the copy engine reads it
// after the call returned; `busy` is recorded after each upload and waited for (host side,
// only until that copy is done) before the buffer is written again.
struct StagingBuffer {
    void *ptr = nullptr;
    size_t bytes = 0;
    hipEvent_t busy = nullptr;
    bool pending = false;
    int reserve(size_t want);     // also waits for a pending upload
    int mark(hipStream_t stream); // record `busy` after an upload was enqueued
    void release();
};

struct TimedLaunch {
    hipEvent_t start, stop;
    int kind;   // 0 = blind rotation, 1 = key switch
};

}  // namespace tfhe

struct tfhe_secret_key {
    uint32_t magic;
    tfhe_params params;
    std::vector<uint32_t> lwe;    // n bits
    std::vector<uint32_t> trlwe;  // N bits
};

struct tfhe_cloud_key {
    uint32_t magic;
    tfhe_params params;
    std::vector<uint32_t> bk_raw;   // [n][2l][2][N]
    std::vector<uint32_t> ksk_raw;  // [N][t][base-1][n+1]
    // device side
    bool uploaded = false;
    int device = -1;
    uint32_t *d_ksk = nullptr;
    void *d_ksk_tiles = nullptr;    // the same key as int8 operand tiles (t = 8, basebit = 2, n < 512 only)
    double2 *d_bk_fft = nullptr;    // [n][2l][4][N/2]: output o = 2*component + limb
    double2 *d_tables = nullptr;    // twiddle tables
    tfhe::DeviceBuffer ws_gates, ws_ext, ws_wires, ws_outs;
    tfhe::StagingBuffer stage_gates, stage_outs;
    // measurement
    bool profile = false;
    std::vector<tfhe::TimedLaunch> timed;
    double prof_ms[2] = {0, 0};
    uint64_t prof_launches[2] = {0, 0};
    uint64_t prof_gates = 0;
    bool margin = false;
    double *d_margin = nullptr;
    // the last layer call: records, wires of its circuit, slots of the wire pool it ran in, depths
    size_t last_layer_gates = 0, last_layer_wires = 0, last_layer_pool = 0, last_layer_levels = 0;
};

#define TFHE_SK_MAGIC 0x53454b31u
#define TFHE_CK_MAGIC 0x434c4b31u
