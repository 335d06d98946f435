/*
 * tfhe_mi355x.h -- C ABI of the MI355X (gfx950) library for batched bootstrapped
 * TFHE gates and encrypted binary-neural-network layers.
 *
 * The service model is the one of the TAPAS paper (Sec. 2, "Encrypted Prediction
 * as a Service"): the client generates keys and encrypts its input bits, the
 * server -- holding the weights and biases in the clear -- evaluates the layers on
 * ciphertexts, the client decrypts.  All data are bits (Sec. 3, "we assume all
 * data to be binary").  The gate primitive is the bootstrapped binary gate of
 * CGGI that the paper builds on (Sec. 3.1.2); its construction is not described in
 * the paper and follows the public one: pre-combination, modulus switch, blind
 * rotation by TRGSW external products over Z_{2^32}[X]/(X^N+1), sample extraction,
 * LWE key switching.
 *
 * Conventions
 *   - Every function returns 0 on success or a negative tfhe_status; nothing
 *     throws or aborts across this boundary.  tfhe_last_error() returns a
 *     thread-local, NUL-terminated description of the last failure.
 *   - A ciphertext is an LWE sample of n+1 little-endian uint32 words
 *     (a_0 .. a_{n-1}, b); arrays of ciphertexts are flat [count][n+1].
 *   - Pointers marked HOST are ordinary host memory, pointers marked DEVICE are
 *     device memory of the current HIP device (e.g. a torch tensor's data_ptr()).
 *     Ciphertext buffers are always owned by the caller.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Server-side calls enqueue work on it and return without synchronising the
 *     device (except when an internal workspace has to grow, which reallocates);
 *     host arrays they take (gate records, weights, thresholds) are consumed
 *     before the call returns.
 *   - Key objects are opaque, owned by the library, released by tfhe_free_*.
 *     A cloud key carries device workspaces that its calls share: issue the
 *     server-side calls on one cloud key from one thread at a time and on one
 *     stream (the stream orders successive calls; calls on different streams would
 *     race on the workspaces).  An uploaded cloud key holds about 180 MB of device
 *     memory for the keys, up to 1.07 GB for the samples between the two kernels
 *     (4,100 B per gate of the widest launch) and, for the layer calls, a wire pool of
 *     one ciphertext (4 (n+1) bytes) per wire that is alive at the same time (about a
 *     third of the layer's gates; tfhe_last_layer_stats reports it).  A layer of more
 *     than about 50 M gates whose units are lowered independently (every lowering but
 *     the "+1" trick and gate sharing) is evaluated in groups of units, so its pool
 *     stays below about 35 GB whatever its size.
 *   - The GPU path supports N = 1024, k = 1, bk_l = 2, bk_Bgbit <= 10, n <= 1024,
 *     ks_t * ks_basebit <= 24, ks_basebit <= 4; other parameters give TFHE_E_PARAM.
 */
#ifndef TFHE_MI355X_H
#define TFHE_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TFHE_OK = 0,
    TFHE_E_NULL = -1,        /* a required pointer is NULL */
    TFHE_E_PARAM = -2,       /* unsupported or inconsistent parameter / gate record */
    TFHE_E_SIZE = -3,        /* a size or index is out of range */
    TFHE_E_HIP = -4,         /* a HIP runtime call failed (see tfhe_last_error) */
    TFHE_E_ALLOC = -5,       /* host or device allocation failed */
    TFHE_E_KEYMISMATCH = -6  /* objects built from different parameter sets */
} tfhe_status;

/* Scheme parameters.  Noise standard deviations are 2^noise_log2 as real torus
 * elements; the benchmark set is {500, 1024, 1, 2, 10, 8, 2, -15, -25}. */
typedef struct {
    int32_t n;              /* LWE dimension */
    int32_t N;              /* ring degree */
    int32_t k;              /* TRLWE mask polynomials (1) */
    int32_t bk_l;           /* gadget length of the bootstrapping key */
    int32_t bk_Bgbit;       /* log2 of its base */
    int32_t ks_t;           /* key-switch digit count */
    int32_t ks_basebit;     /* log2 of the key-switch base */
    int32_t lwe_noise_log2; /* fresh ciphertexts and key-switching key */
    int32_t bk_noise_log2;  /* bootstrapping key */
} tfhe_params;

typedef struct tfhe_secret_key tfhe_secret_key;
typedef struct tfhe_cloud_key tfhe_cloud_key;

/* Gate opcodes.  The paper's circuits use XNOR, AND, OR (Sec. 4.1.1); the other
 * three come from the same mechanism with different constants. */
enum { TFHE_NAND = 0, TFHE_AND = 1, TFHE_OR = 2, TFHE_NOR = 3, TFHE_XOR = 4, TFHE_XNOR = 5,
       /* The three-input multiplexer of Algorithm 1, MUX(s, a, b) = a if s = 1 and b otherwise
        * (Sec. 4.1.1; "a dedicated implementation in TFHE"): two blind rotations -- AND(s, a) and
        * AND(NOT s, b) -- whose sum plus 1/8 is key-switched once.  In a gate stream it is two
        * consecutive records with the same selector, selector flag and output wire:
        *   {TFHE_MUX, negs, nega, s, a, out}  {TFHE_MUX_ELSE, negs, negb, s, b, out}. */
       TFHE_MUX = 6, TFHE_MUX_ELSE = 7 };

/* One gate of a circuit over a wire array: wires[out] = op(+-wires[in0], +-wires[in1]).
 * neg0 / neg1 = 1 takes that input negated: this is how an XNOR with a plaintext
 * weight bit is applied for free (Sec. 4.1.1, "XNORs ... between encrypted and
 * unencrypted data"). */
typedef struct {
    uint8_t op, neg0, neg1, pad;
    int32_t in0, in1, out;
} tfhe_gate_rec;

/* An output of a lowered layer: a wire (possibly negated) or a noiseless constant. */
typedef struct {
    int32_t wire;   /* wire index, or -1 for a constant */
    int32_t value;  /* wire >= 0: 1 = negate the wire; wire < 0: the constant bit */
} tfhe_out_ref;

const char *tfhe_last_error(void);
void tfhe_default_params(tfhe_params *p);

/* ---- client side (Sec. 2: key generation, encryption, decryption) ------------- */

/* Generate the secret key (LWE key of n bits, ring key of N bits) and the cloud key
 * (bootstrapping key: n TRGSW samples; key-switching key: N * t * (2^basebit - 1) LWE
 * samples) deterministically from `seed`.  Host-only work; the cloud key is uploaded
 * to the current device by the first server-side call or by tfhe_cloud_key_upload.
 * Either output pointer may be NULL to skip that object (ck requires the secret key
 * internally and is still generated). */
int tfhe_keygen(const tfhe_params *p, uint64_t seed, tfhe_secret_key **sk, tfhe_cloud_key **ck);

/* Encrypt nbits bits (HOST uint8, 0/1) into ct_host (HOST, [nbits][n+1]); bit 1 is the
 * torus value 1/8, bit 0 is -1/8; mask and noise come from `seed`. */
int tfhe_encrypt(const tfhe_secret_key *sk, uint64_t seed, const uint8_t *bits, size_t nbits,
                 uint32_t *ct_host);

/* Decrypt: bits[i] = 1 iff the phase b - <a, s> of sample i, read as int32, is positive. */
int tfhe_decrypt(const tfhe_secret_key *sk, const uint32_t *ct_host, size_t nbits, uint8_t *bits);

/* Noiseless ciphertext of a known bit (a = 0, b = +-1/8) into ct_host (HOST, n+1 words). */
int tfhe_trivial(const tfhe_params *p, int bit, uint32_t *ct_host);

/* Raw key material for inspection and storage.  which: */
enum { TFHE_KEY_LWE_SK = 0,   /* uint32[n], from a secret key */
       TFHE_KEY_TRLWE_SK = 1, /* uint32[N], from a secret key */
       TFHE_KEY_BK_RAW = 2,   /* uint32[n][2*l][2][N] (row r = u*l + j; mask, body), cloud key */
       TFHE_KEY_KSK_RAW = 3   /* uint32[N][t][2^basebit - 1][n+1], cloud key */ };
/* With buf == NULL stores the byte length in *len; otherwise copies at most *len bytes
 * to buf (HOST) and fails with TFHE_E_SIZE if *len is too small. */
int tfhe_export_key(const void *key, int which, void *buf, size_t *len);
/* The inverse of tfhe_export_key: build key objects from raw material in the layouts above
 * (HOST arrays, copied).  This is how a server receives the cloud key that a client generated
 * (Sec. 2: the client sends its public evaluation key with the encrypted input).
 * sk is built when sk != NULL and needs lwe_sk (n words, each 0 or 1) and trlwe_sk (N words);
 * ck is built when ck != NULL and needs bk_raw and ksk_raw.  Lengths are implied by *p. */
int tfhe_import_keys(const tfhe_params *p, const uint32_t *lwe_sk, const uint32_t *trlwe_sk,
                     const uint32_t *bk_raw, const uint32_t *ksk_raw, tfhe_secret_key **sk,
                     tfhe_cloud_key **ck);
int tfhe_get_params(const void *key, int is_cloud_key, tfhe_params *out);

void tfhe_free_secret_key(tfhe_secret_key *sk);
void tfhe_free_cloud_key(tfhe_cloud_key *ck);
/* Releases arrays returned by the bnn_*_lower functions. */
void tfhe_free_buffer(void *p);

/* ---- server side --------------------------------------------------------------- */

/* Copy the cloud key to the current device and precompute the transform-domain
 * bootstrapping key.  Idempotent; synchronises the device. */
int tfhe_cloud_key_upload(tfhe_cloud_key *ck);

/* count independent bootstrapped gates of one kind: out[i] = op(a[i], b[i]).
 * a, b, out: DEVICE [count][n+1].  out may be the same buffer as a or b (exactly, not
 * shifted).  count == 0 is a no-op. */
int tfhe_gate_batch(tfhe_cloud_key *ck, int op, const uint32_t *a, const uint32_t *b,
                    uint32_t *out, size_t count, void *stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): tfhe_gate_batch with no allocation of any kind inside.
 * The samples between the blind rotation and the key switch -- the one scratch buffer of
 * this path, 4,100 B per gate -- live in a static device array of the library
 * (TFHE_NOALLOC_MAX_GATES x 4,100 B = 16.8 MB per GPU, held until the process ends) instead of
 * the cloud key's growing workspace.  Same arguments, results and aliasing rule as
 * tfhe_gate_batch.  ck must already be uploaded (tfhe_cloud_key_upload, which allocates and
 * looks the array's address up for its device) to the current device; otherwise TFHE_E_PARAM /
 * TFHE_E_HIP.  count > TFHE_NOALLOC_MAX_GATES gives TFHE_E_SIZE and enqueues nothing.
 * Profiling (tfhe_profile_enable) does not cover this call.  All calls on one GPU share the
 * one array: calls that overlap in time on the same GPU (different streams, threads or cloud
 * keys) race; successive calls on one stream do not. */
#define TFHE_NOALLOC_MAX_GATES 4096
int tfhe_gate_batch_noalloc(tfhe_cloud_key *ck, int op, const uint32_t *a, const uint32_t *b,
                            uint32_t *out, size_t count, void *stream);

/* count independent multiplexers: out[i] = s[i] ? a[i] : b[i].  All buffers DEVICE [count][n+1];
 * out may be the same buffer as s, a or b (exactly). */
int tfhe_mux_batch(tfhe_cloud_key *ck, const uint32_t *s, const uint32_t *a, const uint32_t *b,
                   uint32_t *out, size_t count, void *stream);

/* A circuit of mixed gates over a wire array (Sec. 4: "gates at the same level in the
 * tree representation of the circuit can be evaluated in parallel").  gates: HOST,
 * topologically ordered (an input is either never written or written by an earlier
 * record), every wire written at most once.  wires: DEVICE [nwires][n+1], read and
 * written in place.  Gates are grouped by depth and each depth is run as batches. */
int tfhe_gate_stream(tfhe_cloud_key *ck, const tfhe_gate_rec *gates, size_t ngates,
                     uint32_t *wires, size_t nwires, void *stream);

/* Lower a fully connected BNN layer z = sign(Wx + b) (Sec. 3.2) to gates.
 * W: HOST int8 [p][d], entries in {-1, 0, +1} (0 = dropped connection, Sec. 4.3).
 * T: HOST int32 [p], thresholds on the popcount S of the XNORs: output bit = [S >= T]
 *    (step 4 of Sec. 3.2 with T = ceil((d - b) / 2), batch-norm already folded, Sec. 4.1.2);
 *    T == NULL: emit S itself as out_bits little-endian bits per unit (high bits constant 0).
 * Wires 0..d-1 are the inputs, d and d+1 hold noiseless 0 and 1, gate outputs follow.
 * Outputs: *gates (ngates records), *outs (p, or p*out_bits, references), *nwires.
 * The arrays are allocated by the library; release them with tfhe_free_buffer. */
int bnn_dense_lower(int d, const int8_t *W, const int32_t *T, int p, int out_bits,
                    tfhe_gate_rec **gates, size_t *ngates, tfhe_out_ref **outs, size_t *nouts,
                    size_t *nwires);

/* Lowering options (flags of the *_opts entry points). */
enum { TFHE_LOWER_DEFAULT = 0,
       /* comparator exactly as Algorithm 1 prints it: one MUX gate per bit of S with noiseless
        * constants as data inputs (started from o = 1, see bnn_dense_lower), instead of the chain
        * folded to AND / OR gates by the plaintext threshold bits */
       TFHE_LOWER_MUX_COMPARATOR = 1,
       /* the "+1" trick of Sec. 4.2: a unit whose weights are all +-1 sums only the inputs of its
        * rarer weight sign (P over w = +1, or Q over w = -1) and uses the popcount X of all its
        * inputs, computed once and shared by every unit reading the same inputs (a layer's units;
        * a pixel's output channels):  S >= T  <=>  2P - X >= T - |neg|  <=>  X - 2Q >= T - |neg|.
        * The subtraction is an addition of the negated (complemented) bits, the factor 2 a shift,
        * so each unit costs a half-size tree, one ripple-carry adder and the threshold chain.
        * Units with a zero weight are lowered the default way. */
       TFHE_LOWER_PLUS_ONE = 2,
       /* emit a two-input gate only once per (opcode, unordered pair of possibly negated input
        * wires): units that read the same inputs share the lowest levels of their trees, where
        * only the 4 sign patterns of each input pair occur (not in the paper) */
       TFHE_LOWER_SHARE_GATES = 4,
       /* the alternative inner-product circuit of Sec. 4.1.1: sort the XNOR bits in descending
        * order with Batcher's bitonic network of SWAP(a,b) = (OR(a,b), AND(a,b)) and return the bit
        * at position T-1.  The input is padded with noiseless zeros to a power of two; a swap with
        * a known zero needs no gate; only gates the selected position depends on are emitted.
        * Not combinable with TFHE_LOWER_MUX_COMPARATOR / TFHE_LOWER_PLUS_ONE; ignored when T is NULL. */
       TFHE_LOWER_SORTING_NETWORK = 8 };
int bnn_dense_lower_opts(int d, const int8_t *W, const int32_t *T, int p, int out_bits, uint32_t flags,
                         tfhe_gate_rec **gates, size_t *ngates, tfhe_out_ref **outs, size_t *nouts,
                         size_t *nwires);
int bnn_dense_encrypted_opts(tfhe_cloud_key *ck, const uint32_t *x, int d, const int8_t *W,
                             const int32_t *T, int p, uint32_t *out, int out_bits, uint32_t flags,
                             void *stream);

/* Same for a convolution (Sec. 4: "fully connected, convolutional").  x is [C][H][Wd];
 * K: HOST int8 [O][C][kh][kw]; T: HOST int32 [O] (one threshold per output channel).
 * Output pixel (o, y, x) sums the taps (c, ky, kx) in row-major order; a tap outside the
 * image reads the noiseless-0 wire.  outs has O*Ho*Wo entries, Ho = (H + 2 pad - kh)/stride + 1. */
int bnn_conv_lower(int C, int H, int Wd, const int8_t *K, int O, int kh, int kw, int stride,
                   int pad, const int32_t *T, tfhe_gate_rec **gates, size_t *ngates,
                   tfhe_out_ref **outs, size_t *nouts, size_t *nwires);

int bnn_conv_lower_opts(int C, int H, int Wd, const int8_t *K, int O, int kh, int kw, int stride,
                        int pad, const int32_t *T, uint32_t flags, tfhe_gate_rec **gates, size_t *ngates,
                        tfhe_out_ref **outs, size_t *nouts, size_t *nwires);
int bnn_conv_encrypted_opts(tfhe_cloud_key *ck, const uint32_t *x, int C, int H, int Wd,
                            const int8_t *K, int O, int kh, int kw, int stride, int pad,
                            const int32_t *T, uint32_t *out, uint32_t flags, void *stream);

/* Evaluate a fully connected layer on ciphertexts.  x: DEVICE [d][n+1]; W, T as above (HOST);
 * out: DEVICE [p][n+1] (T given) or [p*out_bits][n+1] (T == NULL). */
int bnn_dense_encrypted(tfhe_cloud_key *ck, const uint32_t *x, int d, const int8_t *W,
                        const int32_t *T, int p, uint32_t *out, int out_bits, void *stream);

/* Evaluate a convolution layer on ciphertexts.  x: DEVICE [C*H*Wd][n+1];
 * out: DEVICE [O*Ho*Wo][n+1]. */
int bnn_conv_encrypted(tfhe_cloud_key *ck, const uint32_t *x, int C, int H, int Wd,
                       const int8_t *K, int O, int kh, int kw, int stride, int pad,
                       const int32_t *T, uint32_t *out, void *stream);

/* ---- measurement helpers ---------------------------------------------------------- */

/* Kernel-time accounting of server-side calls on a cloud key: when enabled, every blind
 * rotation and key-switch launch is bracketed by HIP events on the call's stream.
 * tfhe_profile_read synchronises the stream's events and returns accumulated milliseconds
 * and launch counts since the last reset.  Recording never waits for the device. */
typedef struct {
    double blind_rotate_ms, key_switch_ms;
    uint64_t blind_rotate_launches, key_switch_launches, gates;
} tfhe_profile;
int tfhe_profile_enable(tfhe_cloud_key *ck, int on);
int tfhe_profile_read(tfhe_cloud_key *ck, tfhe_profile *out, int reset);

/* The schedule a layer call runs, as a host-side function: sort a lowered circuit by depth and
 * rename its wires to slots of a pool in which a slot is reused once the last depth that reads
 * its wire has run.  Wires 0 .. n_fixed-1 (inputs and the two constants) and the wires referenced
 * by outs keep their slots; outs (HOST, nouts entries) is rewritten in place to slot numbers.
 * *planned (release with tfhe_free_buffer) receives the ngates records in depth order with slot
 * numbers: evaluating them in that order, depth by depth, on a pool of *pool_wires slots gives
 * the circuit's outputs.  Same validation and errors as tfhe_gate_stream. */
int tfhe_plan_wire_pool(const tfhe_gate_rec *gates, size_t ngates, size_t nwires, size_t n_fixed,
                        tfhe_out_ref *outs, size_t nouts, tfhe_gate_rec **planned, size_t *pool_wires,
                        size_t *depths);

/* Shape of the circuit that the last bnn_*_encrypted call on this cloud key ran: gate records,
 * wires of the lowered circuit (inputs, the two constants, one per gate), slots of the wire pool
 * it was evaluated in (a slot is reused once the last depth reading its wire has run; this is
 * the device memory the call needed, 4 (n+1) bytes per slot), and circuit depths (= kernel
 * pairs when no depth is wider than a launch).  For a layer evaluated in groups of units, gates
 * and wires are totals, pool_wires and depths the largest of any group. */
typedef struct {
    uint64_t gates, circuit_wires, pool_wires, depths;
} tfhe_layer_stats;
int tfhe_last_layer_stats(const tfhe_cloud_key *ck, tfhe_layer_stats *out);

/* Double-precision rate (TFLOP/s) that a register-resident FMA loop sustains on the key's device:
 * the measured ceiling of the vector ALU that the blind rotation's transforms run on, to set
 * beside the published peak.  Runs three short launches on `stream` and waits for them. */
int tfhe_measure_fp64_peak(tfhe_cloud_key *ck, void *stream, double *tflops);

/* Largest distance from an integer seen by the blind-rotation kernel when it rounds the
 * inverse transform of its exact split-integer products (0.5 would be a wrong result).
 * Collected only while enabled (slower); read synchronises the device. */
int tfhe_rounding_margin_enable(tfhe_cloud_key *ck, int on);
int tfhe_rounding_margin_read(tfhe_cloud_key *ck, double *max_fraction);

#ifdef __cplusplus
}
#endif
#endif /* TFHE_MI355X_H */
