// Server-side host code: cloud-key upload, batched gate calls, the gate-stream executor.
//
// The data-parallel structure is the one the TAPAS paper points out (Sec. 4): gates at the
// same depth of a circuit are independent, and so are the output units of a layer (Sec. 5.3).
// The executor sorts a circuit by depth and runs each depth as large batches of the two
// kernels (blind rotation, then key switch) on the caller's stream, without host
// synchronisation in between.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "common.h"
#include "kernels.h"

namespace tfhe {

int DeviceBuffer::reserve(size_t want) {
    if (want <= bytes) return TFHE_OK;
    if (ptr) { TFHE_HIP(hipFree(ptr)); ptr = nullptr; bytes = 0; }
    // grow geometrically so that a sequence of slightly larger calls does not reallocate each time
    size_t grown = std::max(want, bytes + bytes / 2);
    hipError_t e = hipMalloc(&ptr, grown);
    if (e != hipSuccess && grown != want) { grown = want; e = hipMalloc(&ptr, grown); }
    if (e != hipSuccess) {
        ptr = nullptr;
        return set_error(TFHE_E_ALLOC, "hipMalloc of %zu bytes failed: %s", grown, hipGetErrorString(e));
    }
    bytes = grown;
    return TFHE_OK;
}

void DeviceBuffer::release() {
    if (ptr) (void)hipFree(ptr);
    ptr = nullptr;
    bytes = 0;
}

int StagingBuffer::reserve(size_t want) {
    if (pending) { TFHE_HIP(hipEventSynchronize(busy)); pending = false; }
    if (want <= bytes) return TFHE_OK;
    if (ptr) { TFHE_HIP(hipHostFree(ptr)); ptr = nullptr; bytes = 0; }
    const size_t grown = std::max(want, bytes + bytes / 2);
    hipError_t e = hipHostMalloc(&ptr, grown, hipHostMallocDefault);
    if (e != hipSuccess) {
        ptr = nullptr;
        return set_error(TFHE_E_ALLOC, "hipHostMalloc of %zu bytes failed: %s", grown, hipGetErrorString(e));
    }
    bytes = grown;
    return TFHE_OK;
}

int StagingBuffer::mark(hipStream_t stream) {
    if (!busy) TFHE_HIP(hipEventCreateWithFlags(&busy, hipEventDisableTiming));
    TFHE_HIP(hipEventRecord(busy, stream));
    pending = true;
    return TFHE_OK;
}

void StagingBuffer::release() {
    if (pending) (void)hipEventSynchronize(busy);
    if (busy) (void)hipEventDestroy(busy);
    if (ptr) (void)hipHostFree(ptr);
    ptr = nullptr; bytes = 0; busy = nullptr; pending = false;
}

namespace {

// Launch items per kernel pair.  A launch ends with CUs idling until its slowest workgroup is done
// (about one gate latency), so a circuit level should be one launch where it can; the limit only
// bounds the extract workspace (4,100 B per item: 1.07 GB).
// an environment override, read once (function-local statics initialise thread-safely)
long env_long(const char *name, long fallback) {
    const char *e = getenv(name);
    return e ? atol(e) : fallback;
}

size_t chunk_gates() {
    static const size_t cached = [] {
        const long v = env_long("TFHE_CHUNK_GATES", 0);
        return v >= 2 ? (size_t)v & ~(size_t)1 : (size_t)1 << 18;
    }();
    return cached;
}

int gates_per_group() {
    static const int cached = [] {
        const long v = env_long("TFHE_GATES_PER_GROUP", 1);
        return (v >= 1 && v <= 3) ? (int)v : 1;
    }();
    return cached;
}

// Gates per key-switch workgroup: large batches amortise the 49 MB key over 16 gates; small
// batches (the deep, narrow levels of a circuit) need many short workgroups instead.
int key_switch_group(size_t count) {
    static const int forced = (int)env_long("TFHE_KS_GROUP", 0);
    if (forced > 0) return forced;
    if (count >= 8192) return 16;
    if (count >= 2048) return 4;
    return 1;
}

// Batches from which the key switch runs as an int8 contraction on the matrix cores: all of them
// (small batches split each gate's mask words over several workgroups; 16 gates take 0.035 ms
// against 0.086 ms of the gather kernels, 256 gates 0.065 against 0.42 ms).  The gather kernels
// remain for parameter sets the matrix kernel does not cover.
int key_switch_matrix(size_t count) {
    static const long threshold = env_long("TFHE_KS_MATRIX_FROM", 1);
    return threshold > 0 && count >= (size_t)threshold;
}

int check_cloud_key(const tfhe_cloud_key *ck) {
    if (!ck) return set_error(TFHE_E_NULL, "cloud key is NULL");
    if (ck->magic != TFHE_CK_MAGIC) return set_error(TFHE_E_PARAM, "not a cloud key");
    return check_params_gpu(&ck->params);
}

int begin_timed(tfhe_cloud_key *ck, int kind, hipStream_t stream, TimedLaunch &tl) {
    tl.kind = kind;
    TFHE_HIP(hipEventCreate(&tl.start));
    TFHE_HIP(hipEventCreate(&tl.stop));
    TFHE_HIP(hipEventRecord(tl.start, stream));
    (void)ck;
    return TFHE_OK;
}

// Add the finished event pairs to the totals and release them.
int drain_timed(tfhe_cloud_key *ck) {
    for (auto &tl : ck->timed) {
        TFHE_HIP(hipEventSynchronize(tl.stop));
        float ms = 0;
        TFHE_HIP(hipEventElapsedTime(&ms, tl.start, tl.stop));
        ck->prof_ms[tl.kind] += ms;
        ck->prof_launches[tl.kind] += 1;
        (void)hipEventDestroy(tl.start);
        (void)hipEventDestroy(tl.stop);
    }
    ck->timed.clear();
    return TFHE_OK;
}

int end_timed(tfhe_cloud_key *ck, hipStream_t stream, TimedLaunch &tl) {
    TFHE_HIP(hipEventRecord(tl.stop, stream));
    ck->timed.push_back(tl);
    // a caller that never reads the profile must not pile up events: fold them in now and then
    // (this waits for the launches so far; profiling is a measurement mode)
    if (ck->timed.size() >= 4096) return drain_timed(ck);
    return TFHE_OK;
}

// One batch of `count` gates: blind rotation into the extract workspace, then key switch.
// `count` counts launch items: a multiplexer is two of them (its two blind rotations).
// `ext` is the [count][N+1] buffer of extracted samples between the two kernels (NULL: the
// cloud key's workspace); with timed = false no event is created even in profiling mode.
int run_batch(tfhe_cloud_key *ck, const tfhe_gate_rec *d_recs, int uniform_op, const uint32_t *in0,
              const uint32_t *in1, const uint32_t *in1_alt, uint32_t *out, size_t count, bool has_mux,
              hipStream_t stream, uint32_t *ext = nullptr, bool timed = true) {
    const tfhe_params &P = ck->params;
    BlindRotateArgs br{};
    br.recs = d_recs; br.uniform_op = uniform_op; br.in0 = in0; br.in1 = in1; br.in1_alt = in1_alt;
    br.ext = ext ? ext : (uint32_t *)ck->ws_ext.ptr; br.count = count;
    br.bk_fft = ck->d_bk_fft; br.tables = ck->d_tables; br.n = P.n; br.bgbit = P.bk_Bgbit;
    br.margin = ck->margin ? ck->d_margin : nullptr;
    KeySwitchArgs ks{};
    ks.ext = br.ext; ks.recs = d_recs; ks.out = out; ks.count = count; ks.ksk = ck->d_ksk;
    ks.n = P.n; ks.t = P.ks_t; ks.basebit = P.ks_basebit; ks.stride = (P.n + 2) & ~1;
    ks.group = key_switch_group(count);
    ks.ksk_tiles = ck->d_ksk_tiles;
    ks.matrix = key_switch_matrix(count);
    // few gates (the deep, narrow levels of a circuit): spread each gate over several
    // workgroups so that the whole chip works on the batch
    ks.splits = 1;
    if (ks.group == 1) {
        static const int forced = (int)env_long("TFHE_KS_SPLITS", 0);
        if (forced > 0) ks.splits = forced;
        else while (ks.splits < 16 && count * ks.splits < 4096) ks.splits *= 2;
    }
    ks.uniform_mux = !d_recs && uniform_op == TFHE_MUX;

    TimedLaunch tl{};
    const bool profile = ck->profile && timed;
    if (profile) if (int rc = begin_timed(ck, 0, stream, tl)) return rc;
    if (int rc = launch_blind_rotate(br, gates_per_group(), stream)) return rc;
    if (profile) if (int rc = end_timed(ck, stream, tl)) return rc;
    if (has_mux) if (int rc = launch_mux_combine(br.ext, d_recs, count, stream)) return rc;
    if (profile) if (int rc = begin_timed(ck, 1, stream, tl)) return rc;
    if (int rc = launch_key_switch(ks, stream)) return rc;
    if (profile) if (int rc = end_timed(ck, stream, tl)) return rc;
    if (profile) ck->prof_gates += count;
    return TFHE_OK;
}

}  // namespace

// Evaluate host gate records (validated, any order within the topological constraint) on device wires.
int run_gate_stream(tfhe_cloud_key *ck, const tfhe_gate_rec *gates, size_t ngates, uint32_t *wires,
                    size_t nwires, hipStream_t stream) {
    if (ngates == 0) return TFHE_OK;
    if (ngates > (size_t)INT32_MAX || nwires > (size_t)INT32_MAX)
        return set_error(TFHE_E_SIZE, "too many gates or wires");
    // writer of each wire; an input must be produced by an earlier record or by nobody.  The
    // second record of a multiplexer shares its output with the first and is not a writer.
    std::vector<int32_t> writer(nwires, -1);
    for (size_t g = 0; g < ngates; ++g) {
        const tfhe_gate_rec &r = gates[g];
        if (r.op > TFHE_MUX_ELSE || r.neg0 > 1 || r.neg1 > 1)
            return set_error(TFHE_E_PARAM, "gate %zu: bad opcode or flag", g);
        if (r.in0 < 0 || r.in1 < 0 || r.out < 0 || (size_t)r.in0 >= nwires || (size_t)r.in1 >= nwires ||
            (size_t)r.out >= nwires)
            return set_error(TFHE_E_SIZE, "gate %zu: wire index out of range", g);
        if (r.op == TFHE_MUX) {
            if (g + 1 >= ngates || gates[g + 1].op != TFHE_MUX_ELSE || gates[g + 1].in0 != r.in0 ||
                gates[g + 1].out != r.out || gates[g + 1].neg0 != r.neg0)
                return set_error(TFHE_E_PARAM, "gate %zu: TFHE_MUX must be followed by its TFHE_MUX_ELSE "
                                               "with the same selector, selector flag and output", g);
        } else if (r.op == TFHE_MUX_ELSE) {
            if (g == 0 || gates[g - 1].op != TFHE_MUX)
                return set_error(TFHE_E_PARAM, "gate %zu: TFHE_MUX_ELSE without its TFHE_MUX", g);
            continue;
        }
        if (writer[r.out] >= 0) return set_error(TFHE_E_PARAM, "gate %zu: wire %d written twice", g, r.out);
        writer[r.out] = (int32_t)g;
    }
    std::vector<int32_t> level(ngates);
    std::vector<int32_t> depth(nwires, 0);
    int32_t max_level = 0;
    bool any_mux = false;
    for (size_t g = 0; g < ngates; ++g) {
        const tfhe_gate_rec &r = gates[g];
        if (r.op == TFHE_MUX_ELSE) { level[g] = level[g - 1]; continue; }
        const int32_t self = (int32_t)g;
        if (writer[r.in0] >= self || writer[r.in1] >= self)
            return set_error(TFHE_E_PARAM, "gate %zu reads a wire written by itself or a later record", g);
        int32_t lv = 1 + std::max(depth[r.in0], depth[r.in1]);
        if (r.op == TFHE_MUX) {
            any_mux = true;
            if (writer[gates[g + 1].in1] >= self)
                return set_error(TFHE_E_PARAM, "gate %zu reads a wire written by itself or a later record", g + 1);
            lv = std::max(lv, 1 + depth[gates[g + 1].in1]);
        }
        level[g] = lv;
        depth[r.out] = lv;
        max_level = std::max(max_level, lv);
    }
    // counting sort by depth
    std::vector<size_t> start(max_level + 2, 0);
    for (size_t g = 0; g < ngates; ++g) ++start[level[g] + 1];
    for (int32_t l = 1; l <= max_level + 1; ++l) start[l] += start[l - 1];
    // sorted records go through a pinned staging buffer: the upload is ordered on the stream and
    // the call does not wait for it (nor for anything queued before it)
    if (int rc = ck->stage_gates.reserve(ngates * sizeof(tfhe_gate_rec))) return rc;
    tfhe_gate_rec *sorted = (tfhe_gate_rec *)ck->stage_gates.ptr;
    {
        std::vector<size_t> at(start.begin(), start.end());
        for (size_t g = 0; g < ngates; ++g) sorted[at[level[g]]++] = gates[g];
    }
    if (int rc = ck->ws_gates.reserve(ngates * sizeof(tfhe_gate_rec))) return rc;
    const size_t kChunkGates = chunk_gates();
    size_t biggest = 0;
    for (int32_t l = 1; l <= max_level; ++l) biggest = std::max(biggest, std::min(kChunkGates, start[l + 1] - start[l]));
    if (int rc = ck->ws_ext.reserve(biggest * (size_t)(ck->params.N + 1) * sizeof(uint32_t))) return rc;
    TFHE_HIP(hipMemcpyAsync(ck->ws_gates.ptr, sorted, ngates * sizeof(tfhe_gate_rec), hipMemcpyHostToDevice,
                            stream));
    if (int rc = ck->stage_gates.mark(stream)) return rc;
    const tfhe_gate_rec *d_recs = (const tfhe_gate_rec *)ck->ws_gates.ptr;
    for (int32_t l = 1; l <= max_level; ++l) {
        for (size_t at = start[l]; at < start[l + 1];) {
            size_t cnt = std::min(kChunkGates, start[l + 1] - at);
            if (sorted[at + cnt - 1].op == TFHE_MUX) --cnt;      // keep the two halves in one batch
            if (int rc = run_batch(ck, d_recs + at, 0, wires, wires, wires, wires, cnt, any_mux, stream)) return rc;
            at += cnt;
        }
    }
    return TFHE_OK;
}

void release_device_keys(tfhe_cloud_key *ck) {
    if (ck->d_ksk) (void)hipFree(ck->d_ksk);
    if (ck->d_ksk_tiles) (void)hipFree(ck->d_ksk_tiles);
    if (ck->d_bk_fft) (void)hipFree(ck->d_bk_fft);
    if (ck->d_tables) (void)hipFree(ck->d_tables);
    if (ck->d_margin) (void)hipFree(ck->d_margin);
    ck->d_ksk = nullptr; ck->d_ksk_tiles = nullptr; ck->d_bk_fft = nullptr; ck->d_tables = nullptr;
    ck->d_margin = nullptr;
    ck->uploaded = false;
}

int ensure_uploaded(tfhe_cloud_key *ck) {
    if (int rc = check_cloud_key(ck)) return rc;
    if (ck->uploaded) return TFHE_OK;
    return tfhe_cloud_key_upload(ck);
}

}  // namespace tfhe

using namespace tfhe;

extern "C" {

static int tfhe_cloud_key_upload_impl(tfhe_cloud_key *ck) {
    if (int rc = check_cloud_key(ck)) return rc;
    if (ck->uploaded) return TFHE_OK;
    const tfhe_params &P = ck->params;
    int count = 0;
    TFHE_HIP(hipGetDeviceCount(&count));
    if (count < 1) return set_error(TFHE_E_HIP, "no HIP device");
    TFHE_HIP(hipGetDevice(&ck->device));
    release_device_keys(ck);          // an earlier attempt may have failed half-way

    // twiddle table psi^j = exp(i pi j / 1024), j < 2048, evaluated in extended precision
    std::vector<double2> tables(2048);
    const long double pi = 3.14159265358979323846264338327950288L;
    for (int j = 0; j < 2048; ++j)
        tables[j] = make_double2((double)cosl(pi * j / 1024), (double)sinl(pi * j / 1024));
    TFHE_HIP(hipMalloc((void **)&ck->d_tables, tables.size() * sizeof(double2)));
    TFHE_HIP(hipMemcpy(ck->d_tables, tables.data(), tables.size() * sizeof(double2), hipMemcpyHostToDevice));

    // key-switching key: rows padded to an even word count (8-byte aligned rows), plus one zero
    // row (what digit 0 reads in the one-gate-per-workgroup kernel)
    const size_t row = (size_t)P.n + 1, stride = (row + 1) & ~(size_t)1, rows = ksk_rows(P);
    TFHE_HIP(hipMalloc((void **)&ck->d_ksk, (rows + 1) * stride * sizeof(uint32_t)));
    TFHE_HIP(hipMemset(ck->d_ksk, 0, (rows + 1) * stride * sizeof(uint32_t)));
    TFHE_HIP(hipMemcpy2D(ck->d_ksk, stride * sizeof(uint32_t), ck->ksk_raw.data(), row * sizeof(uint32_t),
                         row * sizeof(uint32_t), rows, hipMemcpyHostToDevice));

    if (P.ks_t == 8 && P.ks_basebit == 2 && P.N == 1024 && P.n + 1 <= 512) {
        TFHE_HIP(hipMalloc(&ck->d_ksk_tiles, ksk_tiles_bytes()));
        if (int rc = launch_ksk_to_tiles(ck->d_ksk, (int)stride, (int)row, ck->d_ksk_tiles, nullptr)) return rc;
    }

    // bootstrapping key: raw to device, transform on device, raw copy released
    struct RawKey {               // released on every way out
        DeviceBuffer buf;
        ~RawKey() { buf.release(); }
    } raw;
    const size_t bk_bytes = ck->bk_raw.size() * sizeof(uint32_t);
    if (int rc = raw.buf.reserve(bk_bytes)) return rc;
    TFHE_HIP(hipMemcpy(raw.buf.ptr, ck->bk_raw.data(), bk_bytes, hipMemcpyHostToDevice));
    const size_t fft_words = (size_t)P.n * 16 * 512;
    TFHE_HIP(hipMalloc((void **)&ck->d_bk_fft, fft_words * sizeof(double2)));
    if (int rc = launch_bk_to_spectrum((const uint32_t *)raw.buf.ptr, ck->d_bk_fft, ck->d_tables, P.n, nullptr))
        return rc;
    TFHE_HIP(hipDeviceSynchronize());

    TFHE_HIP(hipMalloc((void **)&ck->d_margin, sizeof(double)));
    TFHE_HIP(hipMemset(ck->d_margin, 0, sizeof(double)));
    if (int rc = prepare_kernels()) return rc;
    ck->uploaded = true;
    return TFHE_OK;
}

int tfhe_cloud_key_upload(tfhe_cloud_key *ck) {
    return tfhe::guarded([&]() -> int { return tfhe_cloud_key_upload_impl(ck); });
}

void tfhe_free_cloud_key(tfhe_cloud_key *ck) {
    if (!ck || ck->magic != TFHE_CK_MAGIC) return;
    if (ck->uploaded) (void)hipDeviceSynchronize();
    release_device_keys(ck);          // also what a failed upload left behind
    for (auto &tl : ck->timed) { (void)hipEventDestroy(tl.start); (void)hipEventDestroy(tl.stop); }
    ck->ws_gates.release(); ck->ws_ext.release(); ck->ws_wires.release(); ck->ws_outs.release();
    ck->stage_gates.release(); ck->stage_outs.release();
    ck->magic = 0;
    delete ck;
}

static int tfhe_gate_batch_impl(tfhe_cloud_key *ck, int op, const uint32_t *a, const uint32_t *b, uint32_t *out,
                    size_t count, void *stream) {
    if (int rc = ensure_uploaded(ck)) return rc;
    if (op < TFHE_NAND || op > TFHE_XNOR)
        return set_error(TFHE_E_PARAM, "unknown two-input gate opcode %d (multiplexers: tfhe_mux_batch)", op);
    if (count == 0) return TFHE_OK;
    if (!a || !b || !out) return set_error(TFHE_E_NULL, "NULL ciphertext buffer");
    const size_t words = (size_t)ck->params.n + 1;
    const size_t kChunkGates = chunk_gates();
    const size_t biggest = std::min(kChunkGates, count);
    if (int rc = ck->ws_ext.reserve(biggest * (size_t)(ck->params.N + 1) * sizeof(uint32_t))) return rc;
    for (size_t at = 0; at < count; at += kChunkGates) {
        const size_t cnt = std::min(kChunkGates, count - at);
        if (int rc = run_batch(ck, nullptr, op, a + at * words, b + at * words, nullptr, out + at * words, cnt,
                               false, (hipStream_t)stream))
            return rc;
    }
    return TFHE_OK;
}

int tfhe_gate_batch(tfhe_cloud_key *ck, int op, const uint32_t *a, const uint32_t *b, uint32_t *out,
                    size_t count, void *stream) {
    return tfhe::guarded([&]() -> int { return tfhe_gate_batch_impl(ck, op, a, b, out, count, stream); });
}

// The same gates with no allocation anywhere on the way: the samples between the two kernels go
// to the device's static scratch array, whose address prepare_kernels() looked up at upload.
static int tfhe_gate_batch_noalloc_impl(tfhe_cloud_key *ck, int op, const uint32_t *a, const uint32_t *b,
                                        uint32_t *out, size_t count, void *stream) {
    if (int rc = check_cloud_key(ck)) return rc;
    if (!ck->uploaded)
        return set_error(TFHE_E_PARAM, "tfhe_gate_batch_noalloc needs an uploaded cloud key "
                                       "(call tfhe_cloud_key_upload first: the upload allocates)");
    if (op < TFHE_NAND || op > TFHE_XNOR) return set_error(TFHE_E_PARAM, "unknown two-input gate opcode %d", op);
    if (count > static_scratch_gates())
        return set_error(TFHE_E_SIZE, "tfhe_gate_batch_noalloc takes at most %zu gates per call, got %zu",
                         static_scratch_gates(), count);
    if (count == 0) return TFHE_OK;
    if (!a || !b || !out) return set_error(TFHE_E_NULL, "NULL ciphertext buffer");
    uint32_t *ext = static_scratch_ptr();
    if (!ext) return set_error(TFHE_E_HIP, "the cloud key was uploaded to another device than the current one");
    return run_batch(ck, nullptr, op, a, b, nullptr, out, count, false, (hipStream_t)stream, ext, false);
}

int tfhe_gate_batch_noalloc(tfhe_cloud_key *ck, int op, const uint32_t *a, const uint32_t *b, uint32_t *out,
                            size_t count, void *stream) {
    return tfhe::guarded([&]() -> int { return tfhe_gate_batch_noalloc_impl(ck, op, a, b, out, count, stream); });
}

static int tfhe_mux_batch_impl(tfhe_cloud_key *ck, const uint32_t *s, const uint32_t *a, const uint32_t *b, uint32_t *out,
                   size_t count, void *stream) {
    if (int rc = ensure_uploaded(ck)) return rc;
    if (count == 0) return TFHE_OK;
    if (!s || !a || !b || !out) return set_error(TFHE_E_NULL, "NULL ciphertext buffer");
    const size_t words = (size_t)ck->params.n + 1;
    const size_t per_batch = chunk_gates() / 2;        // two launch items per multiplexer
    const size_t biggest = 2 * std::min(per_batch, count);
    if (int rc = ck->ws_ext.reserve(biggest * (size_t)(ck->params.N + 1) * sizeof(uint32_t))) return rc;
    for (size_t at = 0; at < count; at += per_batch) {
        const size_t cnt = std::min(per_batch, count - at);
        if (int rc = run_batch(ck, nullptr, TFHE_MUX, s + at * words, a + at * words, b + at * words,
                               out + at * words, 2 * cnt, true, (hipStream_t)stream))
            return rc;
    }
    return TFHE_OK;
}

int tfhe_mux_batch(tfhe_cloud_key *ck, const uint32_t *s, const uint32_t *a, const uint32_t *b, uint32_t *out,
                   size_t count, void *stream) {
    return tfhe::guarded([&]() -> int { return tfhe_mux_batch_impl(ck, s, a, b, out, count, stream); });
}

static int tfhe_gate_stream_impl(tfhe_cloud_key *ck, const tfhe_gate_rec *gates, size_t ngates, uint32_t *wires,
                     size_t nwires, void *stream) {
    if (int rc = ensure_uploaded(ck)) return rc;
    if (ngates == 0) return TFHE_OK;
    if (!gates || !wires) return set_error(TFHE_E_NULL, "NULL gates or wires");
    return run_gate_stream(ck, gates, ngates, wires, nwires, (hipStream_t)stream);
}

int tfhe_gate_stream(tfhe_cloud_key *ck, const tfhe_gate_rec *gates, size_t ngates, uint32_t *wires,
                     size_t nwires, void *stream) {
    return tfhe::guarded([&]() -> int { return tfhe_gate_stream_impl(ck, gates, ngates, wires, nwires, stream); });
}

int tfhe_profile_enable(tfhe_cloud_key *ck, int on) {
    if (int rc = check_cloud_key(ck)) return rc;
    ck->profile = on != 0;
    return TFHE_OK;
}

static int tfhe_profile_read_impl(tfhe_cloud_key *ck, tfhe_profile *out, int reset) {
    if (int rc = check_cloud_key(ck)) return rc;
    if (!out) return set_error(TFHE_E_NULL, "NULL profile output");
    if (int rc = drain_timed(ck)) return rc;
    out->blind_rotate_ms = ck->prof_ms[0];
    out->key_switch_ms = ck->prof_ms[1];
    out->blind_rotate_launches = ck->prof_launches[0];
    out->key_switch_launches = ck->prof_launches[1];
    out->gates = ck->prof_gates;
    if (reset) {
        ck->prof_ms[0] = ck->prof_ms[1] = 0;
        ck->prof_launches[0] = ck->prof_launches[1] = 0;
        ck->prof_gates = 0;
    }
    return TFHE_OK;
}

int tfhe_profile_read(tfhe_cloud_key *ck, tfhe_profile *out, int reset) {
    return tfhe::guarded([&]() -> int { return tfhe_profile_read_impl(ck, out, reset); });
}

int tfhe_rounding_margin_enable(tfhe_cloud_key *ck, int on) {
    if (int rc = ensure_uploaded(ck)) return rc;
    ck->margin = on != 0;
    if (on) TFHE_HIP(hipMemset(ck->d_margin, 0, sizeof(double)));
    return TFHE_OK;
}

int tfhe_rounding_margin_read(tfhe_cloud_key *ck, double *max_fraction) {
    if (int rc = ensure_uploaded(ck)) return rc;
    if (!max_fraction) return set_error(TFHE_E_NULL, "NULL output");
    TFHE_HIP(hipDeviceSynchronize());
    TFHE_HIP(hipMemcpy(max_fraction, ck->d_margin, sizeof(double), hipMemcpyDeviceToHost));
    return TFHE_OK;
}

}  // extern "C"
