// Launchers of the gfx950 kernels (kernels.hip), called by the host executor.
#pragma once
#include "common.h"

namespace tfhe {

struct BlindRotateArgs {
    const tfhe_gate_rec *recs;   // device; NULL: gate i reads in0[i], in1[i] with uniform_op
    int uniform_op;
    const uint32_t *in0, *in1;   // device wire arrays the records index into
    const uint32_t *in1_alt;     // uniform TFHE_MUX only: launch item 2g is AND(in0[g], in1[g]),
                                 // item 2g+1 is AND(NOT in0[g], in1_alt[g])
    uint32_t *ext;               // device [count][1025]: extracted samples
    size_t count;
    const double2 *bk_fft;       // device [n][4][4][512]
    const double2 *tables;       // device [2048]: exp(i pi j / 1024)
    int n, bgbit;
    double *margin;              // device, optional: largest rounding distance seen
};

struct KeySwitchArgs {
    const uint32_t *ext;         // device [count][1025]
    const tfhe_gate_rec *recs;   // device; NULL: gate i writes out[i]
    uint32_t *out;               // device wire array
    size_t count;
    const uint32_t *ksk;         // device [1024][t][2^basebit - 1][stride] plus one zero row
    int n, t, basebit;
    int uniform_mux;             // recs == NULL: items come in pairs, item 2g carries the sum and writes out[g]
    int splits;                  // gather kernel: workgroups sharing one gate's mask words (power of two)
    int stride;                  // words per key row on the device: n+1 rounded up to even, pad = 0
    const void *ksk_tiles;       // device, optional: the key as signed-byte tiles for the matrix-core kernel
    int matrix;                  // use the matrix-core kernel (needs ksk_tiles, t = 8, basebit = 2, n + 1 <= 512)
};

size_t blind_rotate_lds_bytes();
int launch_bk_to_spectrum(const uint32_t *bk_raw, double2 *bk_fft, const double2 *tables, int n,
                          hipStream_t stream);
int launch_blind_rotate(const BlindRotateArgs &a, hipStream_t stream);
int launch_key_switch(const KeySwitchArgs &a, hipStream_t stream);
// the key-switching key (device, padded rows) as int8 operand tiles; `tiles` holds ksk_tiles_bytes()
size_t ksk_tiles_bytes();
int launch_ksk_to_tiles(const uint32_t *ksk, int stride, int words, void *tiles, hipStream_t stream);
// ext[e] += ext[e+1]; ext[e].body += 1/8 for every first half e of a multiplexer
int launch_mux_combine(uint32_t *ext, const tfhe_gate_rec *recs, size_t count, hipStream_t stream);
int launch_gather_outputs(const uint32_t *wires, const tfhe_out_ref *refs, uint32_t *out, size_t count,
                          int words, hipStream_t stream);
// per-device set-up at key upload: kernel attributes, address of the static scratch array
int prepare_kernels();
// the static scratch of the current device (NULL before prepare_kernels ran on it) and the
// number of extracted samples ([1025] words each) it holds
uint32_t *static_scratch_ptr();
size_t static_scratch_gates();
// achieved TFLOP/s of a register-resident FP64 FMA loop on the current device (synchronises `stream`)
int measure_fp64_fma_peak(hipStream_t stream, double *sink, double *tflops);
int launch_fill_trivial(uint32_t *ct, int words, int bit, hipStream_t stream);

}  // namespace tfhe
