// C ABI of libapms: argument validation, launch planning, deferred-error
// bookkeeping.  Every entry point validates on the host before touching HIP.

#include "../../include/apms.h"

#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <mutex>
#include <new>

#include "apms_launch.h"
#include "apms_topk.h"

// APMS_GATHER_AUTO: gathers 1..kTuneSamples of a context are timed, cycling through the kTuneForms candidate
// forms (gather 0 pays for loading the kernels and is left out).
constexpr int kTuneForms = 3;        // split; fused with the worker kernel's occupancy cap; fused without it
constexpr int kTuneSamples = 2 * kTuneForms;

struct apms_ctx {
    int64_t d = 0;
    int32_t n = 0;
    int64_t L = 0;
    int64_t C = 0;
    int device = APMS_DEVICE_NONE;
    int32_t w_tiles_per_chunk = 0, w_tiles_per_block = 0, w_blocks_per_chunk = 0;    // apms_compress
    int32_t s_tiles_per_chunk = 0, s_tiles_per_block = 0, s_blocks_per_chunk = 0;    // apms_server_reduce
    int32_t a_tiles_per_chunk = 0;                                                   // apms_apply
    int32_t lds_pad[APMS_KERNEL_COUNT] = {};    // per APMS_KERNEL_*: unused dynamic LDS that caps occupancy
    // device scratch (owned)
    double* w_partials = nullptr;     // [n*C][w_tiles_per_chunk] (sized for 1 tile per block)
    double* s_partials = nullptr;     // [C][s_tiles_per_chunk]
    float* w_pending = nullptr;       // [n*C] scales of the u parked in the worker error buffer
    float* s_pending = nullptr;       // [C]   same for the server error buffer
    float* g_pending = nullptr;       // [C]   server scales of a gather that has not been carried out yet
    apms::TopkScratch topk = {};                // selection scratch of the top-k compressor, allocated by
                                                // apms_topk_reserve
    int64_t topk_bytes = 0;                     // its size so far
    int64_t scratch_bytes = 0;
    // deferral bookkeeping (host side, follows call order = stream order)
    const void* pending_werr = nullptr;       // error buffers that hold u instead of delta
    const void* pending_serr = nullptr;
    bool pending_m_topk = false;              // ... by apms_topk_apply: the momentum is the server's list below, decoded
    const uint32_t* pending_sidx = nullptr;   //     (the caller's arrays, which have to stay as they are meanwhile)
    const float* pending_sval = nullptr;
    int64_t pending_gather_K = 0;
    bool pending_werr_topk = false;           // ... left so by a top-k call (kept positions still in, see TopkScratch.keep)
    bool pending_serr_topk = false;           //     rather than by a 1-bit call (context scales w_pending / s_pending)
    const void* pending_m = nullptr;          // momentum buffer whose gather is still to be written ...
    const uint32_t* pending_spacked = nullptr;  // ... from these sign words (caller's buffer) and g_pending
    int deferral = 0;                         // APMS_DEFER_* flags
    int gather_mode = APMS_GATHER_AUTO;       // how a pending gather is carried out by apms_compress
    // APMS_GATHER_AUTO: the first calls time both forms with events on the caller's stream, read back without
    // waiting by a later call (see pick_gather_form)
    hipEvent_t tune_ev[kTuneSamples][2] = {};
    int tune_calls = 0;                       // gathers carried out so far while undecided
    int tune_choice = -1;                     // index of the candidate form once decided
    float tune_ms[kTuneForms] = {};           // best time seen per candidate form (reported by apms_get_plan)
    int last_hip = 0;
};

// Scratch of apms_server_reduce_static, the entry point for callers that cannot allocate: one copy per GPU
// the library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and copies get the device address static_scratch() returns.
static __device__ __align__(256) unsigned char scratch[APMS_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each device, once resolved

// Device address of the static scratch array on `device`, which must be the current device.  Resolved once
// per device; allocates nothing.
hipError_t static_scratch(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

// Measured on MI355X: the worker kernel streams best with one tile per (short-lived) workgroup, the
// server kernel with a few.
constexpr int32_t kDefaultCompressTiles = 1;
constexpr int32_t kDefaultServerTiles = 4;
constexpr int64_t kMaxGrid = 0x7fffffff;
// Unused dynamic LDS per workgroup, by kernel (compress, server, apply, finalize, warm-up); APMS_PAD_AUTO for
// the worker kernel means "by variant": measured on MI355X, the variant that also writes the gathered
// momentum (two write streams) can gain from 2 workgroups per CU (see gather_form), the variants with one
// write stream run fastest uncapped.  The warm-up kernel (n + 3 read streams) streams fastest with 2
// workgroups (8 waves) per CU, the small-tile kernels with as many as fit.
constexpr int32_t kDefaultLdsPad[APMS_KERNEL_COUNT] = {APMS_PAD_AUTO, 0, 0, 0, 64 * 1024};

struct Range {
    const void* p;
    int64_t bytes;
};

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

bool overlap(const Range& a, const Range& b) {
    if (a.bytes <= 0 || b.bytes <= 0) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a.p), b0 = reinterpret_cast<uintptr_t>(b.p);
    return a0 < b0 + static_cast<uintptr_t>(b.bytes) && b0 < a0 + static_cast<uintptr_t>(a.bytes);
}

// null -> EINVAL, misaligned -> EALIGN, overlapping -> EALIAS; empty arrays (d == 0) are not looked at
int check_arrays(const Range* r, int count) {
    for (int i = 0; i < count; ++i)
        if (r[i].bytes > 0 && !r[i].p) return APMS_EINVAL;
    for (int i = 0; i < count; ++i)
        if (r[i].bytes > 0 && misaligned(r[i].p)) return APMS_EALIGN;
    for (int i = 0; i < count; ++i)
        for (int j = i + 1; j < count; ++j)
            if (overlap(r[i], r[j])) return APMS_EALIAS;
    return APMS_OK;
}

bool unit_interval(float b) { return b >= 0.0f && b < 1.0f; }   // false for NaN

int32_t ceil_div32(int64_t a, int64_t b) { return static_cast<int32_t>((a + b - 1) / b); }

void plan_blocks(apms_ctx* c) {
    c->w_blocks_per_chunk = c->w_tiles_per_chunk ? ceil_div32(c->w_tiles_per_chunk, c->w_tiles_per_block) : 0;
    c->s_blocks_per_chunk = c->s_tiles_per_chunk ? ceil_div32(c->s_tiles_per_chunk, c->s_tiles_per_block) : 0;
}

apms::Geometry geometry(const apms_ctx* c) {
    apms::Geometry g;
    g.d = c->d;
    g.L = c->L;
    g.n = c->n;
    g.C = static_cast<int32_t>(c->C);
    return g;
}

int hip_fail(apms_ctx* c, hipError_t e) {
    c->last_hip = static_cast<int>(e);
    return e == hipErrorOutOfMemory ? APMS_ENOMEM : APMS_EHIP;
}

// Makes the context's device current for the duration of a call.
struct DeviceScope {
    int prev = -1;
    bool switched = false;
    hipError_t err = hipSuccess;
    explicit DeviceScope(int device) {
        err = hipGetDevice(&prev);
        if (err == hipSuccess && prev != device) {
            err = hipSetDevice(device);
            switched = (err == hipSuccess);
        }
    }
    ~DeviceScope() {
        if (switched) (void)hipSetDevice(prev);
    }
};

void clear_pending_gather(apms_ctx* c) {
    c->pending_m = nullptr;
    c->pending_m_topk = false;
    c->pending_spacked = nullptr;
    c->pending_sidx = nullptr;
    c->pending_sval = nullptr;
    c->pending_gather_K = 0;
}

void free_topk_scratch(apms_ctx* c) {
    void* arrays[] = {c->topk.hist, c->topk.state, c->topk.guess, c->topk.last_T, c->topk.keep, c->topk.near, c->topk.gather_offsets,
                      c->topk.tile_counts, c->topk.tile_split, c->topk.slots};
    for (void* a : arrays)
        if (a) (void)hipFree(a);
    c->topk = {};
    c->topk_bytes = 0;
}

// Allocates the top-k scratch (see TopkScratch) with slots for K_max kept elements per chunk; called by
// apms_topk_reserve only (a set-up call: it may allocate, free and synchronise).  The device must be current.
// Every array is fully written by the kernels before they read it, except guess, which is filled here.
hipError_t reserve_topk_scratch(apms_ctx* c, int64_t K_max) {
    const int64_t pairs = static_cast<int64_t>(c->n) * c->C;
    const int64_t tiles = pairs * apms::tiles_per_chunk(geometry(c), apms::kTopkTile);
    const int64_t guesses = pairs + c->C;                     // the worker call's pairs, then the server call's chunks
    const int64_t fixed = (pairs * (apms::kTopkBins + apms::kTopkStateWords + 2 * apms::kTopkNearCap) + 4 * guesses) * 4 +
                          2 * tiles * 4 + tiles / c->n * 4;
    const int32_t want = apms::topk_slots_for(K_max, c->L);
    if (c->topk.slots && c->topk.slots_per_tile >= want) return hipSuccess;
    hipError_t e = hipDeviceSynchronize();                     // kernels of earlier calls may still use the scratch
    if (e != hipSuccess) return e;
    if (!c->topk.hist) {
        e = hipMalloc(reinterpret_cast<void**>(&c->topk.hist), pairs * apms::kTopkBins * 4);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->topk.state), pairs * apms::kTopkStateWords * 4);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->topk.guess), guesses * 4);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->topk.last_T), guesses * 4);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->topk.keep), guesses * 8);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->topk.near), pairs * apms::kTopkNearCap * 8);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->topk.gather_offsets), tiles / c->n * 4);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->topk.tile_counts), tiles * 4);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->topk.tile_split), tiles * 4);
        if (e != hipSuccess) {
            free_topk_scratch(c);
            return e;
        }
        c->topk_bytes = fixed;
    }
    if (c->topk.slots) {
        e = hipFree(c->topk.slots);
        c->topk.slots = nullptr;
        c->topk.slots_per_tile = 0;
        c->topk_bytes = fixed;
        if (e != hipSuccess) return e;
    }
    const int64_t bytes = tiles * want * static_cast<int64_t>(sizeof(uint2));
    e = hipMalloc(reinterpret_cast<void**>(&c->topk.slots), bytes);
    if (e != hipSuccess) {
        c->topk.slots = nullptr;
        return e;
    }
    // no guess to go by: the slots' size decides how low a guess may be without overflowing them
    e = hipMemset(c->topk.guess, 0xFF, guesses * 4);
    if (e == hipSuccess) e = hipMemset(c->topk.last_T, 0xFF, guesses * 4);
    if (e == hipSuccess) e = hipDeviceSynchronize();           // the fill is on the null stream: done before any caller stream goes on
    if (e != hipSuccess) return e;
    c->topk.slots_per_tile = want;
    c->topk_bytes = fixed + bytes;
    return hipSuccess;
}

// A top-k compute call may run only on scratch that apms_topk_reserve sized for at least this K.
bool topk_reserved_for(const apms_ctx* c, int64_t K) {
    return c->topk.slots != nullptr && c->topk.slots_per_tile >= apms::topk_slots_for(K, c->L);
}

void free_scratch(apms_ctx* c) {
    if (c->w_partials) (void)hipFree(c->w_partials);
    if (c->s_partials) (void)hipFree(c->s_partials);
    if (c->w_pending) (void)hipFree(c->w_pending);
    if (c->s_pending) (void)hipFree(c->s_pending);
    if (c->g_pending) (void)hipFree(c->g_pending);
    free_topk_scratch(c);
    for (auto& pair : c->tune_ev)
        for (hipEvent_t& ev : pair) {
            if (ev) (void)hipEventDestroy(ev);
            ev = nullptr;
        }
    c->w_partials = c->s_partials = nullptr;
    c->w_pending = c->s_pending = c->g_pending = nullptr;
}

// Occupancy pads of the worker kernel when the caller leaves them to the library (APMS_PAD_AUTO), from sweeps
// on MI355X with BERT-Large-sized buffers: with a momentum stream of its own (m read, or the gathered m
// written) two workgroups per CU stream best; with error and gradient alone, three.
constexpr int32_t kPadWorkerReadsOrWritesMomentum = 64 * 1024;
constexpr int32_t kPadWorkerNoMomentum = 48 * 1024;

// Candidate forms of a gather-carrying apms_compress: split (0), fused with the worker kernel capped at two
// workgroups per CU (1), fused uncapped (2).  An occupancy pad set by the caller overrides the cap, which
// makes 1 and 2 the same.
struct GatherForm {
    bool fused;
    int32_t pad;       // occupancy pad of the worker kernel in this form
};
GatherForm gather_form(const apms_ctx* c, int index) {
    const int32_t set = c->lds_pad[APMS_KERNEL_COMPRESS];
    if (index == 0) return {false, set != APMS_PAD_AUTO ? set : kPadWorkerNoMomentum};
    return {true, set != APMS_PAD_AUTO ? set : (index == 1 ? kPadWorkerReadsOrWritesMomentum : 0)};
}

// Index of the form the gather of this call takes and, through *sample, the pair of events to bracket it with
// (nullptr: do not time it).  In APMS_GATHER_AUTO the context times its gathers 1..kTuneSamples, cycling
// through the candidate forms, and decides as soon as a later call finds all those events complete; it never
// waits for them.  A stream under graph capture is neither timed nor queried.
int pick_gather_form(apms_ctx* c, hipStream_t s, hipEvent_t** sample) {
    *sample = nullptr;
    if (c->gather_mode != APMS_GATHER_AUTO) return c->gather_mode == APMS_GATHER_FUSED ? 1 : 0;
    if (c->tune_choice >= 0) return c->tune_choice;
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &capture) != hipSuccess || capture != hipStreamCaptureStatusNone) {
        (void)hipGetLastError();
        return 0;
    }
    const int call = c->tune_calls++;
    if (call == 0) return 0;
    if (call <= kTuneSamples) {
        *sample = c->tune_ev[call - 1];
        return (call - 1) % kTuneForms;
    }
    float best[kTuneForms] = {};
    for (int k = 0; k < kTuneSamples; ++k) {
        float ms = 0.0f;
        if (hipEventQuery(c->tune_ev[k][1]) != hipSuccess ||
            hipEventElapsedTime(&ms, c->tune_ev[k][0], c->tune_ev[k][1]) != hipSuccess) {
            (void)hipGetLastError();                           // not ready yet is no error of this call
            return 0;                                          // undecided: ask again at the next gather
        }
        float& b = best[k % kTuneForms];
        if (b == 0.0f || ms < b) b = ms;
    }
    int choice = 0;
    for (int f = 0; f < kTuneForms; ++f) {
        c->tune_ms[f] = best[f];
        if (best[f] < best[choice]) choice = f;
    }
    c->tune_choice = choice;
    return choice;
}

// Common tail of validation: empty problem -> OK (done), validation-only context -> ENODEV.
// Returns 1 when the caller should go on and launch.
int ready_to_launch(const apms_ctx* c, int* status) {
    if (c->d == 0) {
        *status = APMS_OK;
        return 0;
    }
    if (c->device == APMS_DEVICE_NONE) {
        *status = APMS_ENODEV;
        return 0;
    }
    return 1;
}

}  // namespace

extern "C" {

const char* apms_strerror(int status) {
    switch (status) {
        case APMS_OK: return "ok";
        case APMS_EINVAL: return "invalid argument (null pointer or scalar out of range)";
        case APMS_EALIGN: return "array pointer is not 16-byte aligned";
        case APMS_ESHAPE: return "chunk_elems must be a positive multiple of 32 and divide d; at most 4096 workers; grids and top-k list positions must fit 31 bits";
        case APMS_ENOMEM: return "allocation of the context's scratch failed";
        case APMS_EHIP: return "a HIP call failed (see apms_last_hip_error)";
        case APMS_ENODEV: return "validation-only context: no device to run on";
        case APMS_EALIAS: return "array arguments overlap";
        case APMS_ELIMIT: return "the problem needs more than the call's fixed-size scratch holds";
        case APMS_ESTATE: return "the context is not in a state for this call: a buffer is pending in deferred form (call apms_finalize first), or the top-k scratch was not reserved for this K (call apms_topk_reserve)";
        default: return "unknown apms status";
    }
}

int apms_create(apms_ctx** out, int64_t d, int32_t n, int64_t chunk_elems, int device) {
    if (!out) return APMS_EINVAL;
    *out = nullptr;
    if (n < 1 || d < 0 || (device < 0 && device != APMS_DEVICE_NONE)) return APMS_EINVAL;
    if (chunk_elems < 32 || chunk_elems % 32 != 0 || d % chunk_elems != 0) return APMS_ESHAPE;
    if (n > apms::kServerMaxWorkers) return APMS_ESHAPE;     // the server kernel stages one scale per worker in LDS
    const int64_t C = d / chunk_elems;
    // every grid must fit a 1-D launch, every (worker, chunk) index an int32: bound them all by the
    // finest tiling any kernel uses
    constexpr int64_t kMinTile = apms::tile_elems(1);
    const int64_t tiles = (chunk_elems + kMinTile - 1) / kMinTile;
    if (tiles > kMaxGrid || C > kMaxGrid || static_cast<int64_t>(n) * C > kMaxGrid ||
        static_cast<int64_t>(n) * C * tiles > kMaxGrid)
        return APMS_ESHAPE;
    apms_ctx* c = new (std::nothrow) apms_ctx();
    if (!c) return APMS_ENOMEM;
    c->d = d;
    c->n = n;
    c->L = chunk_elems;
    c->C = C;
    c->device = device;
    const apms::Geometry geo = geometry(c);
    c->w_tiles_per_chunk = static_cast<int32_t>(apms::tiles_per_chunk(geo, apms::kCompressTile));
    c->s_tiles_per_chunk = static_cast<int32_t>(apms::tiles_per_chunk(geo, apms::kServerTile));
    c->a_tiles_per_chunk = static_cast<int32_t>(apms::tiles_per_chunk(geo, apms::kApplyTile));
    for (int k = 0; k < APMS_KERNEL_COUNT; ++k) c->lds_pad[k] = kDefaultLdsPad[k];
    c->w_tiles_per_block = kDefaultCompressTiles;
    c->s_tiles_per_block = kDefaultServerTiles;
    plan_blocks(c);
    const int64_t pairs = static_cast<int64_t>(n) * C;
    const int64_t wp = pairs * c->w_tiles_per_chunk * static_cast<int64_t>(sizeof(double));
    const int64_t sp = C * c->s_tiles_per_chunk * static_cast<int64_t>(sizeof(double));
    const int64_t wq = pairs * static_cast<int64_t>(sizeof(float));
    const int64_t sq = C * static_cast<int64_t>(sizeof(float));
    c->scratch_bytes = wp + sp + wq + 2 * sq;
    if (device != APMS_DEVICE_NONE && d > 0) {
        DeviceScope scope(device);
        hipError_t e = scope.err;
        if (e == hipSuccess) e = apms::enable_large_lds_pads();
        void* unused = nullptr;
        if (e == hipSuccess) e = static_scratch(device, &unused);   // so that apms_server_reduce_static finds it resolved
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->w_partials), wp);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->s_partials), sp);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->w_pending), wq);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->s_pending), sq);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c->g_pending), sq);
        for (int k = 0; k < kTuneSamples && e == hipSuccess; ++k)
            for (int j = 0; j < 2 && e == hipSuccess; ++j) e = hipEventCreate(&c->tune_ev[k][j]);
        if (e != hipSuccess) {
            free_scratch(c);
            delete c;
            return e == hipErrorOutOfMemory ? APMS_ENOMEM : APMS_EHIP;
        }
    }
    *out = c;
    return APMS_OK;
}

int apms_destroy(apms_ctx* ctx) {
    if (!ctx) return APMS_OK;
    if (ctx->device != APMS_DEVICE_NONE) {
        DeviceScope scope(ctx->device);
        free_scratch(ctx);
    }
    delete ctx;
    return APMS_OK;
}

int apms_last_hip_error(const apms_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

int apms_get_plan(const apms_ctx* c, apms_plan* plan) {
    if (!c || !plan) return APMS_EINVAL;
    plan->d = c->d;
    plan->n = c->n;
    plan->chunk_elems = c->L;
    plan->chunks = c->C;
    plan->compress_tile_elems = apms::kCompressTile;
    plan->compress_tiles_per_block = c->w_tiles_per_block;
    plan->compress_blocks_per_chunk = c->w_blocks_per_chunk;
    plan->compress_grid = static_cast<int64_t>(c->n) * c->C * c->w_blocks_per_chunk;
    plan->server_tile_elems = apms::kServerTile;
    plan->server_tiles_per_block = c->s_tiles_per_block;
    plan->server_blocks_per_chunk = c->s_blocks_per_chunk;
    plan->server_grid = c->C * c->s_blocks_per_chunk;
    plan->apply_tile_elems = apms::kApplyTile;
    plan->apply_grid = c->C * c->a_tiles_per_chunk * c->n;
    plan->scratch_bytes = c->scratch_bytes;
    plan->topk_scratch_bytes = c->topk_bytes;
    plan->gather_mode = c->gather_mode;
    plan->gather_choice = c->gather_mode != APMS_GATHER_AUTO ? c->gather_mode
                          : c->tune_choice < 0 ? -1 : (c->tune_choice == 0 ? APMS_GATHER_SPLIT : APMS_GATHER_FUSED);
    plan->gather_uncapped = (c->gather_mode == APMS_GATHER_AUTO && c->tune_choice == 2) ? 1 : 0;
    for (int f = 0; f < 3; ++f) plan->gather_ms[f] = c->tune_ms[f];
    for (int k = 0; k < 8; ++k) plan->occupancy_pad[k] = k < APMS_KERNEL_COUNT ? c->lds_pad[k] : 0;
    return APMS_OK;
}

int apms_set_tiles_per_block(apms_ctx* c, int32_t compress_tiles, int32_t server_tiles) {
    if (!c || compress_tiles < 0 || server_tiles < 0) return APMS_EINVAL;
    if (compress_tiles) c->w_tiles_per_block = compress_tiles;
    if (server_tiles) c->s_tiles_per_block = server_tiles;
    plan_blocks(c);
    return APMS_OK;
}

int apms_set_occupancy_pad(apms_ctx* c, int kernel, int32_t lds_bytes) {
    if (!c || kernel < 0 || kernel >= APMS_KERNEL_COUNT || lds_bytes > apms::kMaxLdsPad) return APMS_EINVAL;
    if (lds_bytes < 0 && !(lds_bytes == APMS_PAD_AUTO && kernel == APMS_KERNEL_COMPRESS)) return APMS_EINVAL;
    c->lds_pad[kernel] = lds_bytes;
    return APMS_OK;
}

int apms_set_gather_mode(apms_ctx* c, int mode) {
    if (!c || (mode != APMS_GATHER_SPLIT && mode != APMS_GATHER_FUSED && mode != APMS_GATHER_AUTO)) return APMS_EINVAL;
    c->gather_mode = mode;
    c->tune_calls = 0;                                         // APMS_GATHER_AUTO starts measuring afresh
    c->tune_choice = -1;
    for (float& ms : c->tune_ms) ms = 0.0f;
    return APMS_OK;
}

int apms_set_deferral(apms_ctx* c, int flags) {
    if (!c || (flags & ~(APMS_DEFER_ERRORS | APMS_DEFER_GATHER | APMS_IMPLICIT_MOMENTUM)) != 0) return APMS_EINVAL;
    if ((flags & APMS_IMPLICIT_MOMENTUM) && !(flags & APMS_DEFER_GATHER)) return APMS_EINVAL;
    c->deferral = flags;
    return APMS_OK;
}

int apms_finalize(apms_ctx* c, float* worker_err, float* server_err, float* m, void* stream) {
    if (!c) return APMS_EINVAL;
    if ((worker_err && misaligned(worker_err)) || (server_err && misaligned(server_err)) || (m && misaligned(m)))
        return APMS_EALIGN;
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const apms::Geometry geo = geometry(c);
    if (worker_err && c->pending_werr == worker_err) {
        hipError_t e = c->pending_werr_topk
                           ? apms::launch_topk_finalize(geo, /*server=*/false, worker_err, c->topk, s)
                           : apms::launch_finalize(geo, c->n, worker_err, c->w_pending, c->lds_pad[APMS_KERNEL_FINALIZE], s);
        if (e != hipSuccess) return hip_fail(c, e);
        c->pending_werr = nullptr;
        c->pending_werr_topk = false;
    }
    if (server_err && c->pending_serr == server_err) {
        hipError_t e = c->pending_serr_topk
                           ? apms::launch_topk_finalize(geo, /*server=*/true, server_err, c->topk, s)
                           : apms::launch_finalize(geo, 1, server_err, c->s_pending, c->lds_pad[APMS_KERNEL_FINALIZE], s);
        if (e != hipSuccess) return hip_fail(c, e);
        c->pending_serr = nullptr;
        c->pending_serr_topk = false;
    }
    if (m && c->pending_m == m) {
        hipError_t e = c->pending_m_topk
                           ? apms::launch_topk_apply(geo, c->pending_gather_K, c->pending_sidx, c->pending_sval, nullptr,
                                                     nullptr, m, 0.0f, 0.0f, /*write_m=*/true, /*model_step=*/false,
                                                     c->topk, s)
                           : apms::launch_apply(geo, c->pending_spacked, c->g_pending, nullptr, nullptr, m, nullptr,
                                                /*write_m=*/true, /*model_step=*/false, 0.0f, 0.0f,
                                                c->lds_pad[APMS_KERNEL_APPLY], s);
        if (e != hipSuccess) return hip_fail(c, e);
        clear_pending_gather(c);
    }
    return APMS_OK;
}

}  // extern "C"

namespace {

int grad_elem_bytes(int grad_format) {
    switch (grad_format) {
        case apms::kGradF32: return 4;
        case APMS_GRAD_F16:
        case APMS_GRAD_BF16: return 2;
        default: return 0;
    }
}

int warmup_impl(apms_ctx* c, float* x, float* m, float* v, const void* g, int grad_format, float lr, float beta1,
                float beta2, float eps, int64_t t, void* stream) {
    if (!c) return APMS_EINVAL;
    const int gbytes = grad_elem_bytes(grad_format);
    if (!gbytes) return APMS_EINVAL;
    const int64_t vec = c->d * 4;
    const Range r[] = {{x, vec}, {m, vec}, {v, vec}, {g, c->d * gbytes * c->n}};
    if (int rc = check_arrays(r, 4)) return rc;
    if (!unit_interval(beta1) || !unit_interval(beta2) || t < 1 || !(lr == lr) || !(eps == eps))
        return APMS_EINVAL;
    if (c->pending_m && c->pending_m == m) return APMS_ESTATE;   // slice 0 is not final yet
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    const float bc1 = static_cast<float>(1.0 - std::pow(static_cast<double>(beta1), static_cast<double>(t)));
    const float bc2 = static_cast<float>(1.0 - std::pow(static_cast<double>(beta2), static_cast<double>(t)));
    const float inv_n = 1.0f / static_cast<float>(c->n);
    hipError_t e = apms::launch_warmup(c->d, c->n, x, m, v, g, grad_format, lr, beta1, 1.0f - beta1, beta2,
                                       1.0f - beta2, bc1, bc2, eps, inv_n, c->lds_pad[APMS_KERNEL_WARMUP],
                                       static_cast<hipStream_t>(stream));
    return e == hipSuccess ? APMS_OK : hip_fail(c, e);
}

// with_momentum false: APGSqueeze variant, u = g + delta; m is not an argument and a pending gather is
// neither used nor disturbed.
int compress_impl(apms_ctx* c, bool with_momentum, float* m, const void* g, int grad_format, float* worker_err,
                  uint32_t* packed, float* scales, float beta, void* stream) {
    if (!c) return APMS_EINVAL;
    const int gbytes = grad_elem_bytes(grad_format);
    if (!gbytes) return APMS_EINVAL;
    const int64_t all = c->d * 4 * c->n;
    const bool gather = with_momentum && c->pending_m != nullptr;
    const Range r[] = {{g, c->d * gbytes * c->n}, {worker_err, all}, {packed, all / 32}, {scales, c->n * c->C * 4},
                       {m, with_momentum ? all : 0}, {c->pending_spacked, (gather && !c->pending_m_topk) ? c->d / 8 : 0}};
    if (int rc = check_arrays(r, 6)) return rc;
    if (!unit_interval(beta)) return APMS_EINVAL;
    if (c->pending_werr && (c->pending_werr != worker_err || c->pending_werr_topk)) return APMS_ESTATE;
    if (gather && (c->pending_m != m || c->pending_m_topk)) return APMS_ESTATE;   // another buffer, or the top-k path's form
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const apms::Geometry geo = geometry(c);
    const float* prev = c->pending_werr ? c->w_pending : nullptr;
    const int momentum = !with_momentum ? apms::kMomNone : gather ? apms::kMomGather : apms::kMomRead;
    // implicit momentum: the pending gather is consumed without materialising m
    float* m_arg = (gather && (c->deferral & APMS_IMPLICIT_MOMENTUM)) ? nullptr : m;
    hipError_t e = hipSuccess;
    hipEvent_t* sample = nullptr;
    // no gather to write: by variant (reads m: three read streams; no m at all: two)
    int32_t pad = c->lds_pad[APMS_KERNEL_COMPRESS] != APMS_PAD_AUTO ? c->lds_pad[APMS_KERNEL_COMPRESS]
                  : (momentum == apms::kMomRead ? kPadWorkerReadsOrWritesMomentum : kPadWorkerNoMomentum);
    if (gather && m_arg) {
        const GatherForm form = gather_form(c, pick_gather_form(c, s, &sample));
        pad = form.pad;
        if (sample) e = hipEventRecord(sample[0], s);
        if (e == hipSuccess && !form.fused) {
            // the n momentum slices as one fill of its own; the worker kernel then leaves m alone
            e = apms::launch_apply(geo, c->pending_spacked, c->g_pending, nullptr, nullptr, m, nullptr,
                                   /*write_m=*/true, /*model_step=*/false, 0.0f, 0.0f, c->lds_pad[APMS_KERNEL_APPLY], s);
            m_arg = nullptr;
        }
    }
    const bool eager = !(c->deferral & APMS_DEFER_ERRORS);
    // eager errors and a chunk that fits on chip: one pass writes the finished error (its scales have the
    // bits of the two-pass route with one tile per workgroup, so that is the tiling it stands in for)
    const bool onepass = eager && c->L <= apms::kOnePassMaxChunk && c->w_tiles_per_block == 1;
    if (e == hipSuccess && onepass)
        e = apms::launch_compress_onepass(geo, momentum, m_arg, g, grad_format, worker_err, packed, scales,
                                          c->w_pending, prev, gather ? c->pending_spacked : nullptr,
                                          gather ? c->g_pending : nullptr, beta, 1.0f - beta, s);
    if (e == hipSuccess && !onepass)
        e = apms::launch_compress(geo, c->w_tiles_per_block, c->w_blocks_per_chunk, momentum, m_arg, g,
                                  grad_format, worker_err, packed, c->w_partials, prev,
                                  gather ? c->pending_spacked : nullptr, gather ? c->g_pending : nullptr,
                                  beta, 1.0f - beta, pad, s);
    if (e == hipSuccess && sample) e = hipEventRecord(sample[1], s);
    if (e == hipSuccess && !onepass)
        e = apms::launch_scales(static_cast<int64_t>(c->n) * c->C, c->w_blocks_per_chunk, c->L, c->w_partials, scales,
                                c->w_pending, s);
    if (e == hipSuccess && eager && !onepass)
        e = apms::launch_finalize(geo, c->n, worker_err, c->w_pending, c->lds_pad[APMS_KERNEL_FINALIZE], s);
    if (e != hipSuccess) return hip_fail(c, e);
    // every launch of the call is queued: m holds the gathered momentum (unless implicit); deferred, the
    // error buffer holds u and the context its scales
    if (gather) clear_pending_gather(c);
    c->pending_werr = eager ? nullptr : worker_err;
    return APMS_OK;
}

}  // namespace

extern "C" {

int apms_warmup_step(apms_ctx* c, float* x, float* m, float* v, const float* g, float lr, float beta1,
                     float beta2, float eps, int64_t t, void* stream) {
    return warmup_impl(c, x, m, v, g, apms::kGradF32, lr, beta1, beta2, eps, t, stream);
}

int apms_warmup_step_g16(apms_ctx* c, float* x, float* m, float* v, const uint16_t* g, int grad_format, float lr,
                         float beta1, float beta2, float eps, int64_t t, void* stream) {
    if (grad_format != APMS_GRAD_F16 && grad_format != APMS_GRAD_BF16) return APMS_EINVAL;
    return warmup_impl(c, x, m, v, g, grad_format, lr, beta1, beta2, eps, t, stream);
}

int apms_freeze(apms_ctx* c, float* m, float* worker_err, float* server_err, void* stream) {
    if (!c) return APMS_EINVAL;
    const int64_t vec = c->d * 4;
    const Range r[] = {{m, vec * c->n}, {worker_err, vec * c->n}, {server_err, vec}};
    if (int rc = check_arrays(r, 3)) return rc;
    if (c->pending_m && c->pending_m == m) return APMS_ESTATE;   // slice 0 is not final yet
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    hipError_t e = apms::launch_freeze(c->d, c->n, m, worker_err, server_err, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(c, e);
    c->pending_werr = nullptr;
    c->pending_serr = nullptr;
    c->pending_werr_topk = c->pending_serr_topk = false;
    return APMS_OK;
}

int apms_compress(apms_ctx* c, float* m, const float* g, float* worker_err, uint32_t* packed, float* scales,
                  float beta, void* stream) {
    return compress_impl(c, true, m, g, apms::kGradF32, worker_err, packed, scales, beta, stream);
}

int apms_compress_g16(apms_ctx* c, float* m, const uint16_t* g, int grad_format, float* worker_err,
                      uint32_t* packed, float* scales, float beta, void* stream) {
    if (grad_format != APMS_GRAD_F16 && grad_format != APMS_GRAD_BF16) return APMS_EINVAL;
    return compress_impl(c, true, m, g, grad_format, worker_err, packed, scales, beta, stream);
}

int apms_compress_gradient(apms_ctx* c, const void* g, int grad_format, float* worker_err, uint32_t* packed,
                           float* scales, void* stream) {
    return compress_impl(c, false, nullptr, g, grad_format, worker_err, packed, scales, 0.0f, stream);
}

int apms_server_reduce(apms_ctx* c, const uint32_t* packed, const float* scales, float* server_err,
                       uint32_t* spacked, float* sscales, void* stream) {
    if (!c) return APMS_EINVAL;
    const int64_t vec = c->d * 4;
    const Range r[] = {{packed, vec / 32 * c->n}, {scales, c->n * c->C * 4}, {server_err, vec},
                       {spacked, vec / 32}, {sscales, c->C * 4}};
    if (int rc = check_arrays(r, 5)) return rc;
    if (c->pending_serr && (c->pending_serr != server_err || c->pending_serr_topk)) return APMS_ESTATE;
    // a pending gather still needs the sign words at that address
    if (c->pending_m && !c->pending_m_topk && overlap({c->pending_spacked, vec / 32}, {spacked, vec / 32})) return APMS_ESTATE;
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const apms::Geometry geo = geometry(c);
    const float* prev = c->pending_serr ? c->s_pending : nullptr;
    const float inv_n = 1.0f / static_cast<float>(c->n);
    hipError_t e = apms::launch_server_reduce(geo, c->s_tiles_per_block, c->s_blocks_per_chunk, packed, scales,
                                              server_err, spacked, c->s_partials, prev, inv_n,
                                              c->lds_pad[APMS_KERNEL_SERVER], s);
    if (e == hipSuccess) e = apms::launch_scales(c->C, c->s_blocks_per_chunk, c->L, c->s_partials, sscales, c->s_pending, s);
    const bool eager = !(c->deferral & APMS_DEFER_ERRORS);
    if (e == hipSuccess && eager)
        e = apms::launch_finalize(geo, 1, server_err, c->s_pending, c->lds_pad[APMS_KERNEL_FINALIZE], s);
    if (e != hipSuccess) return hip_fail(c, e);
    c->pending_serr = eager ? nullptr : server_err;          // only once every launch of the call is queued
    return APMS_OK;
}

int apms_server_reduce_static(int64_t d, int32_t n, int64_t chunk_elems, const uint32_t* packed, const float* scales,
                              float* server_err, uint32_t* spacked, float* sscales, void* stream) {
    if (n < 1 || d < 0) return APMS_EINVAL;
    if (chunk_elems < 32 || chunk_elems % 32 != 0 || d % chunk_elems != 0) return APMS_ESHAPE;
    if (n > apms::kServerMaxWorkers) return APMS_ESHAPE;
    const int64_t C = d / chunk_elems;
    apms::Geometry geo;
    geo.d = d;
    geo.L = chunk_elems;
    geo.n = n;
    geo.C = static_cast<int32_t>(C);
    const int64_t tiles = C ? apms::tiles_per_chunk(geo, apms::kServerTile) : 0;
    const int64_t blocks_per_chunk = (tiles + kDefaultServerTiles - 1) / kDefaultServerTiles;   // a new context's tiling
    if (C > kMaxGrid || static_cast<int64_t>(n) * C > kMaxGrid || C * blocks_per_chunk > kMaxGrid ||
        C * ((chunk_elems + apms::kFinalizeTile - 1) / apms::kFinalizeTile) > kMaxGrid)
        return APMS_ESHAPE;
    if (C * blocks_per_chunk * static_cast<int64_t>(sizeof(double)) > APMS_STATIC_SCRATCH_BYTES) return APMS_ELIMIT;
    const int64_t vec = d * 4;
    const Range r[] = {{packed, vec / 32 * n}, {scales, n * C * 4}, {server_err, vec}, {spacked, vec / 32}, {sscales, C * 4}};
    if (int rc = check_arrays(r, 5)) return rc;
    if (d == 0) return APMS_OK;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return APMS_EHIP;
    void* base = nullptr;
    if (static_scratch(device, &base) != hipSuccess) return APMS_EHIP;
    double* partials = static_cast<double*>(base);           // every entry is written before it is read
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = apms::launch_server_reduce(geo, kDefaultServerTiles, static_cast<int32_t>(blocks_per_chunk), packed,
                                              scales, server_err, spacked, partials, nullptr,
                                              1.0f / static_cast<float>(n), kDefaultLdsPad[APMS_KERNEL_SERVER], s);
    if (e == hipSuccess)
        e = apms::launch_scales(C, static_cast<int32_t>(blocks_per_chunk), chunk_elems, partials, sscales, nullptr, s);
    if (e == hipSuccess) e = apms::launch_finalize(geo, 1, server_err, sscales, kDefaultLdsPad[APMS_KERNEL_FINALIZE], s);
    return e == hipSuccess ? APMS_OK : APMS_EHIP;
}

int apms_apply(apms_ctx* c, const uint32_t* spacked, const float* sscales, const float* v, float* x, float* m,
               float lr, float eps, void* stream) {
    if (!c) return APMS_EINVAL;
    const int64_t vec = c->d * 4;
    const Range r[] = {{spacked, vec / 32}, {sscales, c->C * 4}, {v, vec}, {x, vec}, {m, vec * c->n}};
    if (int rc = check_arrays(r, 5)) return rc;
    if (!(lr == lr) || !(eps == eps)) return APMS_EINVAL;
    if (c->pending_m && c->pending_m != m) return APMS_ESTATE;
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    const bool defer = (c->deferral & APMS_DEFER_GATHER) != 0;
    hipError_t e = apms::launch_apply(geometry(c), spacked, sscales, v, x, m, c->g_pending, /*write_m=*/!defer,
                                      /*model_step=*/true, lr, eps, c->lds_pad[APMS_KERNEL_APPLY],
                                      static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(c, e);
    // eager: m is final (a gather pending on it from an earlier call is superseded);
    // deferred: m is to be written from these sign words and the saved scales
    clear_pending_gather(c);
    c->pending_m = defer ? m : nullptr;
    c->pending_spacked = defer ? spacked : nullptr;
    return APMS_OK;
}

int apms_apply_gradient(apms_ctx* c, const uint32_t* spacked, const float* sscales, const float* v, float* x,
                        float* m, float lr, float beta, float eps, void* stream) {
    if (!c) return APMS_EINVAL;
    const int64_t vec = c->d * 4;
    const Range r[] = {{spacked, vec / 32}, {sscales, c->C * 4}, {v, vec}, {x, vec}, {m, vec * c->n}};
    if (int rc = check_arrays(r, 5)) return rc;
    if (!(lr == lr) || !(eps == eps) || !unit_interval(beta)) return APMS_EINVAL;
    if (c->pending_m && c->pending_m == m) return APMS_ESTATE;   // m is read here and is not final yet
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    hipError_t e = apms::launch_apply_gradient(geometry(c), spacked, sscales, v, x, m, lr, beta, 1.0f - beta, eps,
                                               c->lds_pad[APMS_KERNEL_APPLY], static_cast<hipStream_t>(stream));
    return e == hipSuccess ? APMS_OK : hip_fail(c, e);
}

// ---- top-k compressor (Section 5.1, second bullet): eager only -------------------------------------

static int topk_shape_ok(const apms_ctx* c, int64_t K) {
    if (c->L > (int64_t{1} << 31)) return APMS_ESHAPE;        // chunk-local indices are 32-bit
    if (K < 1 || K > c->L) return APMS_EINVAL;
    if (K > INT32_MAX) return APMS_ESHAPE;                    // list positions are 32-bit in the kernels
    return APMS_OK;
}

int apms_topk_reserve(apms_ctx* c, int64_t K_max) {
    if (!c) return APMS_EINVAL;
    if (c->d > 0)
        if (int rc = topk_shape_ok(c, K_max)) return rc;
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    const hipError_t e = reserve_topk_scratch(c, K_max);
    return e == hipSuccess ? APMS_OK : hip_fail(c, e);
}

int apms_topk_compress(apms_ctx* c, float* m, const float* g, float* worker_err, uint32_t* idx, float* val,
                       int64_t K, float beta, void* stream) {
    if (!c) return APMS_EINVAL;
    if (c->d > 0)
        if (int rc = topk_shape_ok(c, K)) return rc;
    const int64_t all = c->d * 4 * c->n, lists = c->n * c->C * K * 4;
    const bool gather = c->pending_m != nullptr;
    const int64_t glists = gather ? c->C * c->pending_gather_K * 4 : 0;
    const Range r[] = {{m, all}, {g, all}, {worker_err, all}, {idx, lists}, {val, lists},
                       {c->pending_sidx, glists}, {c->pending_sval, glists}};
    if (int rc = check_arrays(r, 7)) return rc;
    if (!unit_interval(beta)) return APMS_EINVAL;
    // the momentum is read as it is, or is the pending gather of this path on this buffer; the error is final or
    // as a top-k call left it
    if (gather && !(c->pending_m_topk && c->pending_m == m)) return APMS_ESTATE;
    if (c->pending_werr && !(c->pending_werr_topk && c->pending_werr == worker_err)) return APMS_ESTATE;
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    if (!topk_reserved_for(c, K)) return APMS_ESTATE;
    const bool defer = (c->deferral & APMS_DEFER_ERRORS) != 0;
    const apms::TopkGather list = {c->pending_sidx, c->pending_sval, c->pending_gather_K};
    // implicit momentum: the pending gather is consumed without materialising m
    float* m_arg = (gather && (c->deferral & APMS_IMPLICIT_MOMENTUM)) ? nullptr : m;
    hipError_t e = apms::launch_topk_compress(geometry(c), K, m_arg, g, worker_err, idx, val, beta, 1.0f - beta,
                                              c->pending_werr != nullptr, defer, gather ? &list : nullptr, c->topk,
                                              static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(c, e);
    if (gather) clear_pending_gather(c);
    c->pending_werr = defer ? worker_err : nullptr;
    c->pending_werr_topk = defer;
    return APMS_OK;
}

int apms_topk_server_reduce(apms_ctx* c, const uint32_t* idx, const float* val, int64_t K, float* server_err,
                            uint32_t* sidx, float* sval, void* stream) {
    if (!c) return APMS_EINVAL;
    if (c->d > 0)
        if (int rc = topk_shape_ok(c, K)) return rc;
    const int64_t lists = c->n * c->C * K * 4, slists = c->C * K * 4;
    const Range r[] = {{idx, lists}, {val, lists}, {server_err, c->d * 4}, {sidx, slists}, {sval, slists}};
    if (int rc = check_arrays(r, 5)) return rc;
    if (c->pending_serr && !(c->pending_serr_topk && c->pending_serr == server_err)) return APMS_ESTATE;
    // a pending gather still needs the server's list at that address
    if (c->pending_m && c->pending_m_topk) {
        const int64_t held = c->C * c->pending_gather_K * 4;
        if (overlap({c->pending_sidx, held}, {sidx, slists}) || overlap({c->pending_sval, held}, {sval, slists}) ||
            overlap({c->pending_sidx, held}, {sval, slists}) || overlap({c->pending_sval, held}, {sidx, slists}))
            return APMS_ESTATE;
    }
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    if (!topk_reserved_for(c, K)) return APMS_ESTATE;
    const bool defer = (c->deferral & APMS_DEFER_ERRORS) != 0;
    hipError_t e = apms::launch_topk_server_reduce(geometry(c), K, idx, val, server_err, sidx, sval,
                                                   1.0f / static_cast<float>(c->n), c->pending_serr != nullptr, defer,
                                                   c->topk, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(c, e);
    c->pending_serr = defer ? server_err : nullptr;
    c->pending_serr_topk = defer;
    return APMS_OK;
}

int apms_topk_apply(apms_ctx* c, const uint32_t* sidx, const float* sval, int64_t K, const float* v, float* x,
                    float* m, float lr, float eps, void* stream) {
    if (!c) return APMS_EINVAL;
    if (c->d > 0)
        if (int rc = topk_shape_ok(c, K)) return rc;
    const int64_t vec = c->d * 4, slists = c->C * K * 4;
    const Range r[] = {{sidx, slists}, {sval, slists}, {v, vec}, {x, vec}, {m, vec * c->n}};
    if (int rc = check_arrays(r, 5)) return rc;
    if (!(lr == lr) || !(eps == eps)) return APMS_EINVAL;
    if (c->pending_m && c->pending_m != m) return APMS_ESTATE;   // a gather pending on the same buffer is superseded
    int status;
    if (!ready_to_launch(c, &status)) return status;
    DeviceScope scope(c->device);
    if (scope.err != hipSuccess) return hip_fail(c, scope.err);
    if (!topk_reserved_for(c, K)) return APMS_ESTATE;
    const bool defer = (c->deferral & APMS_DEFER_GATHER) != 0;
    hipError_t e = apms::launch_topk_apply(geometry(c), K, sidx, sval, v, x, m, lr, eps, /*write_m=*/!defer,
                                           /*model_step=*/true, c->topk, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(c, e);
    // eager: m is final; deferred: m is to be written from this list, which the caller leaves as it is until then
    clear_pending_gather(c);
    if (defer) {
        c->pending_m = m;
        c->pending_m_topk = true;
        c->pending_sidx = sidx;
        c->pending_sval = sval;
        c->pending_gather_K = K;
    }
    return APMS_OK;
}

}  // extern "C"
