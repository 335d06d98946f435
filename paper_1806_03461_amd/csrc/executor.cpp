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
#include <functional>
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
    // a caller that never reads the profile must not pile up events: now and then fold in the
    // pairs that have already finished, without waiting for any that have not
    if (ck->timed.size() >= 4096 && ck->timed.size() % 1024 == 0) {
        size_t done = 0;
        while (done < ck->timed.size() && hipEventQuery(ck->timed[done].stop) == hipSuccess) {
            float ms = 0;
            TFHE_HIP(hipEventElapsedTime(&ms, ck->timed[done].start, ck->timed[done].stop));
            ck->prof_ms[ck->timed[done].kind] += ms;
            ck->prof_launches[ck->timed[done].kind] += 1;
            (void)hipEventDestroy(ck->timed[done].start);
            (void)hipEventDestroy(ck->timed[done].stop);
            ++done;
        }
        ck->timed.erase(ck->timed.begin(), ck->timed.begin() + (std::ptrdiff_t)done);
    }
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
    ks.ksk_tiles = ck->d_ksk_tiles;
    ks.matrix = key_switch_matrix(count);
    // few gates (the deep, narrow levels of a circuit): spread each gate over several
    // workgroups so that the whole chip works on the batch
    ks.splits = 1;
    {
        static const int forced = (int)env_long("TFHE_KS_SPLITS", 0);
        if (forced > 0) ks.splits = forced;
        else while (ks.splits < 16 && count * ks.splits < 4096) ks.splits *= 2;
    }
    ks.uniform_mux = !d_recs && uniform_op == TFHE_MUX;

    TimedLaunch tl{};
    const bool profile = ck->profile && timed;
    if (profile) if (int rc = begin_timed(ck, 0, stream, tl)) return rc;
    if (int rc = launch_blind_rotate(br, stream)) return rc;
    if (profile) if (int rc = end_timed(ck, stream, tl)) return rc;
    if (has_mux) if (int rc = launch_mux_combine(br.ext, d_recs, count, stream)) return rc;
    if (profile) if (int rc = begin_timed(ck, 1, stream, tl)) return rc;
    if (int rc = launch_key_switch(ks, stream)) return rc;
    if (profile) if (int rc = end_timed(ck, stream, tl)) return rc;
    if (profile) ck->prof_gates += count;
    return TFHE_OK;
}

}  // namespace

namespace {

// Validation and ASAP levels of a topologically ordered gate list.
struct Levels {
    std::vector<int32_t> level;     // per record
    std::vector<size_t> start;      // records of level l occupy sorted positions [start[l], start[l+1])
    int32_t max_level = 0;
    bool any_mux = false;
};

int levelize(const tfhe_gate_rec *gates, size_t ngates, size_t nwires, Levels &lv) {
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
    lv.level.assign(ngates, 0);
    std::vector<int32_t> depth(nwires, 0);
    lv.max_level = 0;
    lv.any_mux = false;
    for (size_t g = 0; g < ngates; ++g) {
        const tfhe_gate_rec &r = gates[g];
        if (r.op == TFHE_MUX_ELSE) { lv.level[g] = lv.level[g - 1]; continue; }
        const int32_t self = (int32_t)g;
        if (writer[r.in0] >= self || writer[r.in1] >= self)
            return set_error(TFHE_E_PARAM, "gate %zu reads a wire written by itself or a later record", g);
        int32_t l = 1 + std::max(depth[r.in0], depth[r.in1]);
        if (r.op == TFHE_MUX) {
            lv.any_mux = true;
            if (writer[gates[g + 1].in1] >= self)
                return set_error(TFHE_E_PARAM, "gate %zu reads a wire written by itself or a later record", g + 1);
            l = std::max(l, 1 + depth[gates[g + 1].in1]);
        }
        lv.level[g] = l;
        depth[r.out] = l;
        lv.max_level = std::max(lv.max_level, l);
    }
    // counting sort by depth
    lv.start.assign((size_t)lv.max_level + 2, 0);
    for (size_t g = 0; g < ngates; ++g) ++lv.start[(size_t)lv.level[g] + 1];
    for (int32_t l = 1; l <= lv.max_level + 1; ++l) lv.start[l] += lv.start[l - 1];
    return TFHE_OK;
}

// The depth-sorted records already sit in the pinned staging buffer: upload them and run one
// kernel pair per depth (in chunks) on the stream.  The upload is ordered on the stream and the
// call does not wait for it (nor for anything queued before it).
int launch_levels(tfhe_cloud_key *ck, size_t ngates, const Levels &lv, uint32_t *wires, hipStream_t stream) {
    const tfhe_gate_rec *sorted = (const tfhe_gate_rec *)ck->stage_gates.ptr;
    if (int rc = ck->ws_gates.reserve(ngates * sizeof(tfhe_gate_rec))) return rc;
    const size_t kChunkGates = chunk_gates();
    size_t biggest = 0;
    for (int32_t l = 1; l <= lv.max_level; ++l)
        biggest = std::max(biggest, std::min(kChunkGates, lv.start[l + 1] - lv.start[l]));
    if (int rc = ck->ws_ext.reserve(biggest * (size_t)(ck->params.N + 1) * sizeof(uint32_t))) return rc;
    TFHE_HIP(hipMemcpyAsync(ck->ws_gates.ptr, sorted, ngates * sizeof(tfhe_gate_rec), hipMemcpyHostToDevice,
                            stream));
    if (int rc = ck->stage_gates.mark(stream)) return rc;
    const tfhe_gate_rec *d_recs = (const tfhe_gate_rec *)ck->ws_gates.ptr;
    for (int32_t l = 1; l <= lv.max_level; ++l) {
        for (size_t at = lv.start[l]; at < lv.start[l + 1];) {
            size_t cnt = std::min(kChunkGates, lv.start[l + 1] - at);
            if (sorted[at + cnt - 1].op == TFHE_MUX) --cnt;      // keep the two halves in one batch
            if (int rc = run_batch(ck, d_recs + at, 0, wires, wires, wires, wires, cnt, lv.any_mux, stream)) return rc;
            at += cnt;
        }
    }
    return TFHE_OK;
}

}  // namespace

// Evaluate host gate records (validated, any order within the topological constraint) on device
// wires that the caller owns: every wire keeps the index the records give it.
int run_gate_stream(tfhe_cloud_key *ck, const tfhe_gate_rec *gates, size_t ngates, uint32_t *wires,
                    size_t nwires, hipStream_t stream) {
    if (ngates == 0) return TFHE_OK;
    Levels lv;
    if (int rc = levelize(gates, ngates, nwires, lv)) return rc;
    if (int rc = ck->stage_gates.reserve(ngates * sizeof(tfhe_gate_rec))) return rc;
    tfhe_gate_rec *sorted = (tfhe_gate_rec *)ck->stage_gates.ptr;
    {
        std::vector<size_t> at(lv.start.begin(), lv.start.end());
        for (size_t g = 0; g < ngates; ++g) sorted[at[lv.level[g]]++] = gates[g];
    }
    return launch_levels(ck, ngates, lv, wires, stream);
}

// Rename the wires of a levelized circuit to slots of a pool: a slot is handed out again once the
// last depth that reads its wire has run (a depth's kernels follow the previous depth's on the
// stream, and a slot freed by depth l is first written by depth l + 1).  Wires 0 .. n_fixed-1
// (a layer's inputs and the two constants) and the wires that `outs` references keep their slots
// to the end.  `sorted` receives the depth-sorted records in slot numbers, `outs` is rewritten
// to slots, *pool_wires is the number of slots used.
int plan_wire_pool(const tfhe_gate_rec *gates, size_t ngates, size_t nwires, size_t n_fixed, const Levels &lv,
                   tfhe_gate_rec *sorted, tfhe_out_ref *outs, size_t nouts, size_t *pool_wires) {
    size_t pool = n_fixed;
    // last depth that reads each wire (its own depth if nothing reads it); outputs never expire
    std::vector<int32_t> last(nwires, 0);
    for (size_t g = 0; g < ngates; ++g) {
        const tfhe_gate_rec &r = gates[g];
        const int32_t l = lv.level[g];
        last[r.in0] = std::max(last[r.in0], l);
        last[r.in1] = std::max(last[r.in1], l);
        last[r.out] = std::max(last[r.out], l);
    }
    for (size_t k = 0; k < nouts; ++k) {
        if (outs[k].wire >= (int64_t)nwires) return set_error(TFHE_E_SIZE, "output %zu: wire index out of range", k);
        if (outs[k].wire >= 0) last[outs[k].wire] = INT32_MAX;
    }
    {
        std::vector<size_t> at(lv.start.begin(), lv.start.end());
        for (size_t g = 0; g < ngates; ++g) sorted[at[lv.level[g]]++] = gates[g];
    }
    std::vector<int32_t> slot(nwires, -1);
    for (size_t w = 0; w < n_fixed && w < nwires; ++w) slot[w] = (int32_t)w;
    std::vector<int32_t> free_slots;
    auto expire = [&](int32_t w, int32_t l) {
        if ((size_t)w >= n_fixed && last[w] == l) { free_slots.push_back(slot[w]); last[w] = -1; }
    };
    for (int32_t l = 1; l <= lv.max_level; ++l) {
        const size_t lo = lv.start[l], hi = lv.start[l + 1];
        for (size_t g = lo; g < hi; ++g) {               // outputs of this depth take slots
            const tfhe_gate_rec &r = sorted[g];
            if (r.op == TFHE_MUX_ELSE) continue;           // shares the output of the record before it
            if ((size_t)r.out < n_fixed) return set_error(TFHE_E_PARAM, "a gate writes a fixed wire");
            if (free_slots.empty()) slot[r.out] = (int32_t)pool++;
            else { slot[r.out] = free_slots.back(); free_slots.pop_back(); }
        }
        for (size_t g = lo; g < hi; ++g) {               // slots freed here serve depth l + 1 onwards
            tfhe_gate_rec &r = sorted[g];
            const int32_t in0 = r.in0, in1 = r.in1, out = r.out;
            if (slot[in0] < 0 || slot[in1] < 0)
                return set_error(TFHE_E_PARAM, "a gate reads a wire that is neither fixed nor written");
            r.in0 = slot[in0]; r.in1 = slot[in1]; r.out = slot[out];
            expire(in0, l); expire(in1, l);
            if (r.op != TFHE_MUX) expire(out, l);           // a multiplexer's output expires with its second record
        }
        if (pool > (size_t)INT32_MAX) return set_error(TFHE_E_SIZE, "wire pool too large");
    }
    for (size_t k = 0; k < nouts; ++k)
        if (outs[k].wire >= 0) {
            if (slot[outs[k].wire] < 0) return set_error(TFHE_E_PARAM, "output %zu references a wire that is never written", k);
            outs[k].wire = slot[outs[k].wire];
        }
    *pool_wires = pool;
    return TFHE_OK;
}

// A layer's circuit on a wire pool the library owns.  `prepare` is called with the pool's size
// (to allocate it and fill its fixed wires) before anything is launched; afterwards `outs`
// refers to slots.
int run_layer_stream(tfhe_cloud_key *ck, const tfhe_gate_rec *gates, size_t ngates, size_t nwires, size_t n_fixed,
                     std::vector<tfhe_out_ref> &outs, hipStream_t stream,
                     const std::function<int(size_t pool_wires, uint32_t **wires)> &prepare) {
    Levels lv;
    size_t pool = n_fixed;
    if (ngates) {
        if (int rc = levelize(gates, ngates, nwires, lv)) return rc;
        if (int rc = ck->stage_gates.reserve(ngates * sizeof(tfhe_gate_rec))) return rc;
        if (int rc = plan_wire_pool(gates, ngates, nwires, n_fixed, lv, (tfhe_gate_rec *)ck->stage_gates.ptr, outs.data(),
                                    outs.size(), &pool))
            return rc;
    }
    ck->last_layer_gates = ngates;
    ck->last_layer_wires = nwires;
    ck->last_layer_pool = pool;
    ck->last_layer_levels = (size_t)lv.max_level;
    uint32_t *wires = nullptr;
    if (int rc = prepare(pool, &wires)) return rc;
    if (ngates == 0) return TFHE_OK;
    return launch_levels(ck, ngates, lv, wires, stream);
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

static int tfhe_plan_wire_pool_impl(const tfhe_gate_rec *gates, size_t ngates, size_t nwires, size_t n_fixed,
                                    tfhe_out_ref *outs, size_t nouts, tfhe_gate_rec **planned, size_t *pool_wires,
                                    size_t *depths) {
    if (!planned || !pool_wires || !depths) return set_error(TFHE_E_NULL, "NULL output pointer");
    if ((ngates && !gates) || (nouts && !outs)) return set_error(TFHE_E_NULL, "NULL gates or outputs");
    if (n_fixed > nwires) return set_error(TFHE_E_SIZE, "more fixed wires than wires");
    Levels lv;
    *planned = (tfhe_gate_rec *)malloc(std::max<size_t>(1, ngates) * sizeof(tfhe_gate_rec));
    if (!*planned) return set_error(TFHE_E_ALLOC, "out of memory");
    *pool_wires = n_fixed;
    *depths = 0;
    if (ngates == 0) return TFHE_OK;
    int rc = levelize(gates, ngates, nwires, lv);
    if (!rc) rc = plan_wire_pool(gates, ngates, nwires, n_fixed, lv, *planned, outs, nouts, pool_wires);
    if (rc) { free(*planned); *planned = nullptr; return rc; }
    *depths = (size_t)lv.max_level;
    return TFHE_OK;
}

int tfhe_plan_wire_pool(const tfhe_gate_rec *gates, size_t ngates, size_t nwires, size_t n_fixed, tfhe_out_ref *outs,
                        size_t nouts, tfhe_gate_rec **planned, size_t *pool_wires, size_t *depths) {
    return tfhe::guarded([&]() -> int {
        return tfhe_plan_wire_pool_impl(gates, ngates, nwires, n_fixed, outs, nouts, planned, pool_wires, depths);
    });
}

int tfhe_last_layer_stats(const tfhe_cloud_key *ck, tfhe_layer_stats *out) {
    if (!ck || ck->magic != TFHE_CK_MAGIC) return set_error(TFHE_E_NULL, "not a cloud key");
    if (!out) return set_error(TFHE_E_NULL, "NULL output");
    out->gates = ck->last_layer_gates;
    out->circuit_wires = ck->last_layer_wires;
    out->pool_wires = ck->last_layer_pool;
    out->depths = ck->last_layer_levels;
    return TFHE_OK;
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

int tfhe_measure_fp64_peak(tfhe_cloud_key *ck, void *stream, double *tflops) {
    return tfhe::guarded([&]() -> int {
        if (int rc = ensure_uploaded(ck)) return rc;
        if (!tflops) return set_error(TFHE_E_NULL, "NULL output");
        return measure_fp64_fma_peak((hipStream_t)stream, ck->d_margin, tflops);
    });
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
