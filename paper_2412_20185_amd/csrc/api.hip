// C ABI of the library (see include/decdec.h): argument checking, the host
// helpers that convert plain code matrices to the private packed layout, and
// the stream choreography of one compensated GEMV.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <new>

#include "../../include/decdec.h"
#include "finalize.h"
#include "kernels.h"
#include "layout.h"

using namespace decdec;

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    (void)hipGetLastError();  // clear the sticky per-thread error
    return DECDEC_EHIP;
}
#define DD_HIP(call)                               \
    do {                                           \
        hipError_t e_ = (call);                    \
        if (e_ != hipSuccess) return hip_fail(e_); \
    } while (0)

int pack_kind(const decdec_desc* d) {
    if (d->wfmt == DECDEC_W_UNIFORM_G128) {
        if (d->wbits == 4) return PACK_U4;
        if (d->wbits == 3) return PACK_U3;
        return -1;
    }
    if (d->wfmt == DECDEC_W_LUT_COL8) return d->wbits == 3 ? PACK_LUT3 : -1;
    return -1;
}

int check_desc(const decdec_desc* d) {
    if (d == nullptr) return DECDEC_EINVAL;
    if (d->K <= 0 || d->N <= 0 || d->K % kGroup != 0 || d->N % kTileCols != 0) return DECDEC_EINVAL;
    if (d->wfmt != DECDEC_W_UNIFORM_G128 && d->wfmt != DECDEC_W_LUT_COL8) return DECDEC_EINVAL;
    if (d->rfmt < DECDEC_R_FP16 || d->rfmt > DECDEC_R_INT8_SYM_COL) return DECDEC_EINVAL;
    if (d->wbits != 3 && d->wbits != 4) return DECDEC_EINVAL;
    if (pack_kind(d) < 0) return DECDEC_EUNSUPPORTED;
    return DECDEC_OK;
}

constexpr int kProfClasses = 4;              // base GEMV, selection, fetch, accumulate
constexpr int kProfEvents = 2 * kProfClasses;  // a (start, stop) pair each

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Residual pointers that have been verified (one attribute query per pointer, ever): an open-addressing
// table over storage the owner supplies, so that looking a pointer up or adding one never allocates.
struct PtrEntry {
    const void* p;      // null: free slot
    size_t avail;       // bytes of the allocation from p to its end; SIZE_MAX when the runtime does not say
    uint8_t in_device;  // 1: device memory, 0: pinned host memory
};

struct PointerTable {
    PtrEntry* e;
    int cap;  // a power of two
    int used;
    long long queries;  // attribute queries made so far

    size_t slot(const void* p) const {
        uint64_t v = reinterpret_cast<uintptr_t>(p);
        v ^= v >> 17;
        v *= 0x9E3779B97F4A7C15ull;
        return (size_t)(v >> 24) & (size_t)(cap - 1);
    }
    const PtrEntry* find(const void* p) const {
        for (size_t i = slot(p), n = 0; n < (size_t)cap; i = (i + 1) & (size_t)(cap - 1), ++n) {
            if (e[i].p == p) return &e[i];
            if (e[i].p == nullptr) return nullptr;
        }
        return nullptr;
    }
    // False when the table is three quarters full: the pointer is then verified again on its next use.
    bool insert(const PtrEntry& x) {
        if (used >= cap - cap / 4) return false;
        size_t i = slot(x.p);
        while (e[i].p != nullptr && e[i].p != x.p) i = (i + 1) & (size_t)(cap - 1);
        if (e[i].p == nullptr) ++used;
        e[i] = x;
        return true;
    }
    void clear() {
        std::memset(e, 0, sizeof(PtrEntry) * (size_t)cap);
        used = 0;
    }
    // Linear probing without tombstones: the entries behind the hole move up.
    void erase(const void* p) {
        size_t i = slot(p);
        for (size_t n = 0; n < (size_t)cap && e[i].p != p; ++n) {
            if (e[i].p == nullptr) return;
            i = (i + 1) & (size_t)(cap - 1);
        }
        if (e[i].p != p) return;
        e[i].p = nullptr;
        --used;
        for (size_t j = (i + 1) & (size_t)(cap - 1); e[j].p != nullptr; j = (j + 1) & (size_t)(cap - 1)) {
            const PtrEntry x = e[j];
            e[j].p = nullptr;
            --used;
            insert(x);
        }
    }
};

constexpr int kWsPointerSlots = 4096;      // a workspace remembers about 3000 residual pointers (a 32-layer model has 224)
constexpr int kStaticPointerSlots = 1024;  // the allocation-free entry point: about 750 per GPU

// What one compensated GEMV needs besides its operands: scratch buffers, options and the table of verified
// residual pointers.  A workspace owns one (buffers from hipMalloc); the allocation-free entry point keeps one
// per GPU whose buffers lie in a static device array.
struct Core {
    int32_t maxK, maxN, maxk;
    int32_t fetch_split;
    int32_t gemv_gpw;
    int32_t gemv_wpb;             // wavefronts per base-GEMV workgroup when it runs as a kernel of its own; 0: built in
    int32_t mode;                 // decdec_mode
    int32_t separate_select;      // 1: selection always runs as a kernel of its own
    int32_t inkernel_accumulate;  // 1: the producers add into the column accumulators (no accumulate kernel)
    int32_t acc_dirty;            // a call failed half-way: clear the accumulators before the next one
    int32_t* idx;        // [maxk]
    void* xsel;          // fp16 [maxk]
    unsigned long long* acc;  // [maxN] per-column fixed-point accumulators, zero between calls
    float* gpart;        // [kMaxGemvSlices][maxN]   partial rows for the separate accumulate kernel:
    float* cpart;        // [kMaxFetchSlices][maxN]  allocated when that path is first switched on
    hipStream_t side;    // null: no second stream (TWO_STREAMS mode unavailable)
    hipEvent_t ev_fork, ev_join;
    PointerTable ptrs;
    // optional kernel timing: per call one (start, stop) event pair per kernel class
    hipEvent_t* prof_ev;  // [prof_cap][kProfEvents]: gemv, select, fetch, accumulate
    uint8_t* prof_mask;   // [prof_cap] bit c: class c was launched and timed
    int32_t prof_cap, prof_used;
};

}  // namespace

struct decdec_ws {
    Core core;
    PtrEntry slots[kWsPointerSlots];
};

extern "C" {

const char* decdec_strerror(int status) {
    switch (status) {
        case DECDEC_OK: return "ok";
        case DECDEC_EINVAL: return "invalid argument";
        case DECDEC_EUNSUPPORTED: return "unsupported format";
        case DECDEC_ENOTPINNED: return "residual pointer is not GPU-visible pinned host memory";
        case DECDEC_EHIP: return "HIP runtime error";
        case DECDEC_ENOMEM: return "out of memory";
        case DECDEC_ETOOLARGE: return "problem exceeds the static scratch buffer of decdec_gemv_static";
        default: return "unknown status";
    }
}

int decdec_last_hip_error(void) { return g_last_hip_error; }

size_t decdec_sc_buffer_bytes(int32_t k) { return k > 0 ? (size_t)k * (4 + 2) : 0; }

size_t decdec_partial_buffer_bytes(int32_t maxN) {
    return maxN > 0 ? (size_t)(kMaxGemvSlices + kMaxFetchSlices) * (size_t)maxN * 4 : 0;
}

// hipMemoryTypeHost / hipMemoryTypeDevice, or -1 for memory the GPU cannot read.
static int residual_memory_type(const void* p) {
    hipPointerAttribute_t at;
    std::memset(&at, 0, sizeof(at));
    const hipError_t e = hipPointerGetAttributes(&at, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    return at.type == hipMemoryTypeHost || at.type == hipMemoryTypeDevice ? (int)at.type : -1;
}

int decdec_check_pinned(const void* p) {
    if (p == nullptr) return DECDEC_EINVAL;
    return residual_memory_type(p) == (int)hipMemoryTypeHost ? DECDEC_OK : DECDEC_ENOTPINNED;
}

int decdec_check_residual_pointer(const void* p) {
    if (p == nullptr) return DECDEC_EINVAL;
    return residual_memory_type(p) >= 0 ? DECDEC_OK : DECDEC_ENOTPINNED;
}

int decdec_ws_create(int32_t maxK, int32_t maxN, int32_t maxk, decdec_ws** out) {
    if (out == nullptr) return DECDEC_EINVAL;
    *out = nullptr;
    if (maxK <= 0 || maxN <= 0 || maxk < 0 || maxk > maxK || maxK > kSelectMaxK) return DECDEC_EINVAL;
    decdec_ws* ws = new (std::nothrow) decdec_ws();
    if (ws == nullptr) return DECDEC_ENOMEM;
    std::memset(ws, 0, sizeof(*ws));
    Core& c = ws->core;
    c.maxK = maxK;
    c.maxN = maxN;
    c.maxk = maxk;
    c.ptrs.e = ws->slots;
    c.ptrs.cap = kWsPointerSlots;
    c.inkernel_accumulate = 1;
    const size_t kk = maxk > 0 ? (size_t)maxk : 1;
    hipError_t e = hipStreamCreateWithFlags(&c.side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c.ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c.ev_join, hipEventDisableTiming);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c.idx), kk * 4);
    if (e == hipSuccess) e = hipMalloc(&c.xsel, kk * 2);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c.acc), (size_t)maxN * 8);
    if (e == hipSuccess) e = hipMemset(c.acc, 0, (size_t)maxN * 8);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        const int rc = e == hipErrorOutOfMemory ? DECDEC_ENOMEM : hip_fail(e);
        (void)hipGetLastError();
        decdec_ws_destroy(ws);
        return rc;
    }
    *out = ws;
    return DECDEC_OK;
}

static void free_profiling(Core& c) {
    if (c.prof_ev) {
        for (int i = 0; i < c.prof_cap * kProfEvents; ++i)
            if (c.prof_ev[i]) (void)hipEventDestroy(c.prof_ev[i]);
        delete[] c.prof_ev;
        delete[] c.prof_mask;
    }
    c.prof_ev = nullptr;
    c.prof_mask = nullptr;
    c.prof_cap = c.prof_used = 0;
}

int decdec_ws_set_profiling(decdec_ws* ws, int32_t capacity) {
    if (ws == nullptr || capacity < 0 || capacity > (1 << 20)) return DECDEC_EINVAL;
    Core& c = ws->core;
    DD_HIP(hipDeviceSynchronize());
    free_profiling(c);
    if (capacity == 0) return DECDEC_OK;
    c.prof_ev = new (std::nothrow) hipEvent_t[(size_t)capacity * kProfEvents]();
    c.prof_mask = new (std::nothrow) uint8_t[capacity]();
    if (c.prof_ev == nullptr || c.prof_mask == nullptr) {
        delete[] c.prof_ev;
        delete[] c.prof_mask;
        c.prof_ev = nullptr;
        c.prof_mask = nullptr;
        return DECDEC_ENOMEM;
    }
    c.prof_cap = capacity;
    for (int i = 0; i < capacity * kProfEvents; ++i) {
        const hipError_t e = hipEventCreate(&c.prof_ev[i]);
        if (e != hipSuccess) {
            free_profiling(c);
            return hip_fail(e);
        }
    }
    return DECDEC_OK;
}

// Per kernel class: summed durations (ms) and launch counts; with per_launch != null also the duration of
// every timed launch of class `cls` in call order (at most per_launch_cap of them, *per_launch_n receives the count).
static int read_profile(Core& c, double* ms_out, int32_t* calls_out, int cls, float* per_launch, int per_launch_cap,
                        int32_t* per_launch_n) {
    double t[kProfClasses] = {0, 0, 0, 0};
    int32_t n[kProfClasses] = {0, 0, 0, 0};
    int32_t listed = 0;
    if (c.prof_ev) {
        DD_HIP(hipDeviceSynchronize());
        for (int i = 0; i < c.prof_used; ++i) {
            hipEvent_t* ev = c.prof_ev + (size_t)i * kProfEvents;
            for (int k = 0; k < kProfClasses; ++k) {
                if (c.prof_mask[i] & (1 << k)) {
                    float ms = 0.f;
                    DD_HIP(hipEventElapsedTime(&ms, ev[2 * k], ev[2 * k + 1]));
                    t[k] += ms;
                    ++n[k];
                    if (k == cls && per_launch != nullptr && listed < per_launch_cap) per_launch[listed++] = ms;
                }
            }
            c.prof_mask[i] = 0;
        }
        c.prof_used = 0;
    }
    for (int k = 0; k < kProfClasses; ++k) {
        if (ms_out) ms_out[k] = t[k];
        if (calls_out) calls_out[k] = n[k];
    }
    if (per_launch_n) *per_launch_n = listed;
    return DECDEC_OK;
}

int decdec_ws_read_profile(decdec_ws* ws, double* ms_out, int32_t* calls_out) {
    if (ws == nullptr) return DECDEC_EINVAL;
    return read_profile(ws->core, ms_out, calls_out, -1, nullptr, 0, nullptr);
}

int decdec_ws_read_profile_launches(decdec_ws* ws, int32_t kernel_class, float* ms_per_launch, int32_t capacity,
                                    int32_t* count_out) {
    if (ws == nullptr || kernel_class < 0 || kernel_class >= kProfClasses || ms_per_launch == nullptr ||
        capacity < 0 || count_out == nullptr)
        return DECDEC_EINVAL;
    return read_profile(ws->core, nullptr, nullptr, kernel_class, ms_per_launch, capacity, count_out);
}

int decdec_ws_destroy(decdec_ws* ws) {
    if (ws == nullptr) return DECDEC_OK;
    Core& c = ws->core;
    free_profiling(c);
    if (c.side) {
        (void)hipStreamSynchronize(c.side);
        (void)hipStreamDestroy(c.side);
    }
    if (c.ev_fork) (void)hipEventDestroy(c.ev_fork);
    if (c.ev_join) (void)hipEventDestroy(c.ev_join);
    if (c.idx) (void)hipFree(c.idx);
    if (c.xsel) (void)hipFree(c.xsel);
    if (c.gpart) (void)hipFree(c.gpart);
    if (c.cpart) (void)hipFree(c.cpart);
    if (c.acc) (void)hipFree(c.acc);
    delete ws;
    return DECDEC_OK;
}

int decdec_ws_last_selection(const decdec_ws* ws, const int32_t** idx_dev, const void** xsel_f16_dev) {
    if (ws == nullptr) return DECDEC_EINVAL;
    if (idx_dev) *idx_dev = ws->core.idx;
    if (xsel_f16_dev) *xsel_f16_dev = ws->core.xsel;
    return DECDEC_OK;
}

int decdec_ws_set_inkernel_accumulate(decdec_ws* ws, int32_t on) {
    if (ws == nullptr || (on != 0 && on != 1)) return DECDEC_EINVAL;
    Core& c = ws->core;
    if (on == 0 && c.gpart == nullptr) {
        // The separate kernel adds fp32 partial rows; they exist only for workspaces that ask for it.
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&c.gpart), (size_t)kMaxGemvSlices * c.maxN * 4);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&c.cpart), (size_t)kMaxFetchSlices * c.maxN * 4);
        if (e != hipSuccess) {
            const int rc = e == hipErrorOutOfMemory ? DECDEC_ENOMEM : hip_fail(e);
            (void)hipGetLastError();
            if (c.gpart) (void)hipFree(c.gpart);
            c.gpart = c.cpart = nullptr;
            return rc;
        }
    }
    c.inkernel_accumulate = on;
    return DECDEC_OK;
}

int decdec_ws_set_mode(decdec_ws* ws, int32_t mode) {
    if (ws == nullptr || mode < DECDEC_MODE_FUSED || mode > DECDEC_MODE_TWO_STREAMS) return DECDEC_EINVAL;
    ws->core.mode = mode;
    return DECDEC_OK;
}

int decdec_ws_set_separate_select(decdec_ws* ws, int32_t on) {
    if (ws == nullptr || (on != 0 && on != 1)) return DECDEC_EINVAL;
    ws->core.separate_select = on;
    return DECDEC_OK;
}

int decdec_ws_set_gemv_split(decdec_ws* ws, int32_t groups_per_wave) {
    if (ws == nullptr || groups_per_wave < 0 || groups_per_wave > 1024) return DECDEC_EINVAL;
    ws->core.gemv_gpw = groups_per_wave;
    return DECDEC_OK;
}

int decdec_ws_set_gemv_waves(decdec_ws* ws, int32_t waves_per_workgroup) {
    if (ws == nullptr || (waves_per_workgroup != 0 && waves_per_workgroup != 4 && waves_per_workgroup != 8 &&
                          waves_per_workgroup != 16))
        return DECDEC_EINVAL;
    ws->core.gemv_wpb = waves_per_workgroup;
    return DECDEC_OK;
}

int decdec_ws_gemv_launch_shape(const decdec_ws* ws, int32_t K, int32_t N_total, int32_t* workgroups,
                                int32_t* threads, int32_t* k_slices) {
    if (ws == nullptr || K <= 0 || K % kGroup != 0 || N_total <= 0 || N_total % kTileCols != 0) return DECDEC_EINVAL;
    const long tiles = N_total / kTileCols;
    const GemvPlan gp = gemv_plan(tiles, K / kGroup, ws->core.gemv_gpw, ws->core.gemv_wpb);
    if (workgroups) *workgroups = (int32_t)(tiles * gp.slices);
    if (threads) *threads = gp.wpb * 64;
    if (k_slices) *k_slices = gp.slices;
    return DECDEC_OK;
}

int decdec_ws_read_selection(const decdec_ws* ws, int32_t k, int32_t* idx_host, void* xsel_f16_host) {
    if (ws == nullptr || k < 0 || k > ws->core.maxk) return DECDEC_EINVAL;
    // The selection may have been written by a kernel on any stream of the caller's: wait for the device.
    DD_HIP(hipDeviceSynchronize());
    if (k == 0) return DECDEC_OK;
    if (idx_host) DD_HIP(hipMemcpy(idx_host, ws->core.idx, (size_t)k * 4, hipMemcpyDeviceToHost));
    if (xsel_f16_host) DD_HIP(hipMemcpy(xsel_f16_host, ws->core.xsel, (size_t)k * 2, hipMemcpyDeviceToHost));
    return DECDEC_OK;
}

int decdec_ws_set_fetch_split(decdec_ws* ws, int32_t row_split) {
    if (ws == nullptr || row_split < 0 || row_split > kMaxFetchSlices * kWavesPerBlock) return DECDEC_EINVAL;
    ws->core.fetch_split = row_split;
    return DECDEC_OK;
}

int decdec_ws_forget_pointer(decdec_ws* ws, const void* p) {
    if (ws == nullptr) return DECDEC_EINVAL;
    if (p == nullptr) {
        ws->core.ptrs.clear();
    } else {
        ws->core.ptrs.erase(p);
    }
    return DECDEC_OK;
}

int64_t decdec_ws_pointer_queries(const decdec_ws* ws) { return ws == nullptr ? -1 : (int64_t)ws->core.ptrs.queries; }

// ------------------------------------------------------------ host helpers

size_t decdec_packed_bytes(const decdec_desc* d) {
    if (check_desc(d) != DECDEC_OK) return 0;
    return (size_t)(d->N / kTileCols) * (size_t)(d->K / kGroup) * (size_t)tile_bytes(pack_kind(d));
}

int decdec_pack_weights(const decdec_desc* d, const uint8_t* codes_KN, void* out_packed) {
    const int rc = check_desc(d);
    if (rc != DECDEC_OK) return rc;
    if (codes_KN == nullptr || out_packed == nullptr) return DECDEC_EINVAL;
    const int kind = pack_kind(d), G = d->K / kGroup, NT = d->N / kTileCols;
    const uint32_t limit = 1u << d->wbits;
    uint8_t* out = static_cast<uint8_t*>(out_packed);
    std::memset(out, 0, decdec_packed_bytes(d));
    for (int nt = 0; nt < NT; ++nt) {
        for (int g = 0; g < G; ++g) {
            uint8_t* tile = out + ((size_t)nt * G + g) * tile_bytes(kind);
            for (int kl = 0; kl < kGroup; ++kl) {
                const CodeSlot slot = code_slot(kind, kl);
                const uint8_t* row = codes_KN + ((size_t)g * kGroup + kl) * d->N + (size_t)nt * kTileCols;
                for (int lane = 0; lane < kTileCols; ++lane) {
                    const uint32_t q = row[lane];
                    if (q >= limit) return DECDEC_EINVAL;
                    for (int r = 0; r < slot.nruns; ++r) {
                        const BitRun br = slot.run[r];
                        uint32_t w;
                        uint8_t* p = tile + word_offset_in_tile(br.word, lane);
                        std::memcpy(&w, p, 4);
                        w |= ((q >> br.code_bit) & ((1u << br.nbits) - 1u)) << br.bit;
                        std::memcpy(p, &w, 4);
                    }
                }
            }
        }
    }
    return DECDEC_OK;
}

int decdec_unpack_weights(const decdec_desc* d, const void* packed, uint8_t* codes_KN) {
    const int rc = check_desc(d);
    if (rc != DECDEC_OK) return rc;
    if (codes_KN == nullptr || packed == nullptr) return DECDEC_EINVAL;
    const int kind = pack_kind(d), G = d->K / kGroup, NT = d->N / kTileCols;
    const uint8_t* in = static_cast<const uint8_t*>(packed);
    for (int nt = 0; nt < NT; ++nt) {
        for (int g = 0; g < G; ++g) {
            const uint8_t* tile = in + ((size_t)nt * G + g) * tile_bytes(kind);
            for (int kl = 0; kl < kGroup; ++kl) {
                const CodeSlot slot = code_slot(kind, kl);
                uint8_t* row = codes_KN + ((size_t)g * kGroup + kl) * d->N + (size_t)nt * kTileCols;
                for (int lane = 0; lane < kTileCols; ++lane) {
                    uint32_t q = 0;
                    for (int r = 0; r < slot.nruns; ++r) {
                        const BitRun br = slot.run[r];
                        uint32_t w;
                        std::memcpy(&w, tile + word_offset_in_tile(br.word, lane), 4);
                        q |= ((w >> br.bit) & ((1u << br.nbits) - 1u)) << br.code_bit;
                    }
                    row[lane] = (uint8_t)q;
                }
            }
        }
    }
    return DECDEC_OK;
}

int decdec_pack_residual_int(int32_t K, int32_t N, int32_t bits, const int8_t* codes_KN, uint8_t* out) {
    if (bits != 2 && bits != 4 && bits != 8) return DECDEC_EUNSUPPORTED;
    const int per_byte = 8 / bits, qmax = (1 << (bits - 1)) - 1;
    if (K <= 0 || N <= 0 || N % (128 / bits) != 0 || codes_KN == nullptr || out == nullptr) return DECDEC_EINVAL;
    const size_t row_bytes = (size_t)N / per_byte;
    for (size_t r = 0; r < (size_t)K; ++r) {
        for (size_t j = 0; j < row_bytes; ++j) {
            unsigned byte = 0;
            for (int i = 0; i < per_byte; ++i) {
                const int q = codes_KN[r * N + j * per_byte + i];
                if (q < -qmax || q > qmax) return DECDEC_EINVAL;
                byte |= ((unsigned)q & ((1u << bits) - 1u)) << (bits * i);
            }
            out[r * row_bytes + j] = (uint8_t)byte;
        }
    }
    return DECDEC_OK;
}

int decdec_pack_residual_int4(int32_t K, int32_t N, const int8_t* codes_KN, uint8_t* out) {
    return decdec_pack_residual_int(K, N, 4, codes_KN, out);
}

// ---------------------------------------------------------------- hot path

int decdec_select_topk(const void* x_f16_dev, int32_t K, int32_t k, int32_t* idx_out_dev, void* xsel_f16_dev,
                       void* stream) {
    if (x_f16_dev == nullptr || K < 8 || K % 8 != 0 || K > kSelectMaxK || k < 0 || k > K) return DECDEC_EINVAL;
    if (!aligned(x_f16_dev, 16)) return DECDEC_EINVAL;
    if (k == 0) return DECDEC_OK;
    if (idx_out_dev == nullptr || !aligned(idx_out_dev, 4) || !aligned(xsel_f16_dev, 2)) return DECDEC_EINVAL;
    DD_HIP(launch_select_topk(x_f16_dev, K, k, idx_out_dev, xsel_f16_dev, static_cast<hipStream_t>(stream)));
    return DECDEC_OK;
}

int decdec_select_bucket(const void* x_f16_dev, int32_t K, int32_t k_chunk, float b0, float b15,
                         int32_t* idx_out_dev, void* xsel_f16_dev, void* stream) {
    if (x_f16_dev == nullptr || K < 1024 || K % 1024 != 0 || k_chunk < 0 || k_chunk > 1024) return DECDEC_EINVAL;
    if (!aligned(x_f16_dev, 16)) return DECDEC_EINVAL;
    if (!(b0 >= b15) || !(b15 >= 0.f)) return DECDEC_EINVAL;  // also rejects NaN
    if (k_chunk == 0) return DECDEC_OK;
    if (idx_out_dev == nullptr || !aligned(idx_out_dev, 4) || !aligned(xsel_f16_dev, 2)) return DECDEC_EINVAL;
    DD_HIP(launch_select_bucket(x_f16_dev, K, k_chunk, b0, b15, idx_out_dev, xsel_f16_dev,
                                static_cast<hipStream_t>(stream)));
    return DECDEC_OK;
}

}  // extern "C"

namespace {

// Looks the residual pointer up; a pointer seen for the first time is verified with one attribute query and
// one address-range query and then remembered.  need: bytes the kernels may read from R on (K rows).
// *in_device: the residuals live in device memory (not over the host link).
int check_residual_cached(PointerTable& tab, const void* R, size_t need, bool* in_device) {
    const PtrEntry* hit = tab.find(R);
    PtrEntry fresh;
    if (hit == nullptr) {
        ++tab.queries;
        const int type = residual_memory_type(R);
        if (type < 0) return DECDEC_ENOTPINNED;
        fresh.p = R;
        fresh.in_device = type == (int)hipMemoryTypeDevice ? 1 : 0;
        fresh.avail = SIZE_MAX;
        void* base = nullptr;
        size_t size = 0;
        if (hipMemGetAddressRange(reinterpret_cast<hipDeviceptr_t*>(&base), &size, const_cast<void*>(R)) == hipSuccess &&
            base != nullptr && size > 0) {
            const uintptr_t end = reinterpret_cast<uintptr_t>(base) + size, at = reinterpret_cast<uintptr_t>(R);
            if (at >= reinterpret_cast<uintptr_t>(base) && at < end) fresh.avail = (size_t)(end - at);
        } else {
            (void)hipGetLastError();  // not every kind of pinned memory reports its range
        }
        (void)tab.insert(fresh);
        hit = &fresh;
    }
    if (need > hit->avail) return DECDEC_EINVAL;  // the allocation is shorter than K rows
    *in_device = hit->in_device != 0;
    return DECDEC_OK;
}

// count linears that share x (and therefore K, the selection, and one launch
// of each kernel).  idx_in/xsel_in: caller-supplied selection or null.
int gemv_common(int32_t count, const decdec_linear* lin, const void* x, int32_t k, const int32_t* idx_in,
                const void* xsel_in, bool have_idx, Core* core, void* stream_v) {
    if (lin == nullptr || count < 1 || count > kMaxMulti || core == nullptr || x == nullptr) return DECDEC_EINVAL;
    Core& c = *core;
    MultiShape sh{};
    GemvOperands gop{};
    FetchOperands fop{};
    void* ys[kMaxMulti] = {};
    sh.n = count;
    const decdec_desc* d0 = lin[0].desc;
    for (int m = 0; m < count; ++m) {
        const decdec_linear& L = lin[m];
        const int rc = check_desc(L.desc);
        if (rc != DECDEC_OK) return rc;
        if (L.desc->K != d0->K) return DECDEC_EINVAL;
        if (L.desc->wbits != d0->wbits || L.desc->wfmt != d0->wfmt || L.desc->rfmt != d0->rfmt)
            return DECDEC_EUNSUPPORTED;
        if (L.Wq_dev == nullptr || L.zeros_or_lut_f16_dev == nullptr || L.y_f16_dev == nullptr) return DECDEC_EINVAL;
        if (L.desc->wfmt == DECDEC_W_UNIFORM_G128 && L.scales_f16_dev == nullptr) return DECDEC_EINVAL;
        // what the kernels' vector and scalar loads assume
        if (!aligned(L.Wq_dev, 16) || !aligned(L.y_f16_dev, 2) || !aligned(L.scales_f16_dev, 2)) return DECDEC_EINVAL;
        if (!aligned(L.zeros_or_lut_f16_dev, L.desc->wfmt == DECDEC_W_LUT_COL8 ? 16 : 2)) return DECDEC_EINVAL;
        sh.N[m] = L.desc->N;
        sh.col0[m + 1] = sh.col0[m] + L.desc->N;
        gop.Wq[m] = L.Wq_dev;
        gop.scales[m] = L.scales_f16_dev;
        gop.zeros_or_lut[m] = L.zeros_or_lut_f16_dev;
        fop.R[m] = L.R_pinned;
        fop.R_scales[m] = L.R_scales_f16_dev;
        ys[m] = L.y_f16_dev;
    }
    sh.K = d0->K;
    if (!aligned(x, 16)) return DECDEC_EINVAL;
    if (sh.K > c.maxK || sh.col0[count] > c.maxN || k < 0 || k > sh.K || k > c.maxk) return DECDEC_EINVAL;
    if (c.mode == DECDEC_MODE_TWO_STREAMS && c.side == nullptr) return DECDEC_EUNSUPPORTED;
    bool residuals_in_hbm = k > 0;  // all of them: the fetch is then bound by HBM latency, not by the host link
    if (k > 0) {
        if (have_idx && (idx_in == nullptr || xsel_in == nullptr || !aligned(idx_in, 4) || !aligned(xsel_in, 2)))
            return DECDEC_EINVAL;
        const int rbits = d0->rfmt == DECDEC_R_FP16 ? 16 : d0->rfmt == DECDEC_R_INT4_SYM_COL ? 4
                        : d0->rfmt == DECDEC_R_INT2_SYM_COL ? 2 : 8;
        for (int m = 0; m < count; ++m) {
            if (lin[m].R_pinned == nullptr || !aligned(lin[m].R_pinned, 16)) return DECDEC_EINVAL;
            if (d0->rfmt != DECDEC_R_FP16 &&
                (lin[m].R_scales_f16_dev == nullptr || !aligned(lin[m].R_scales_f16_dev, 16)))
                return DECDEC_EINVAL;
            if ((size_t)sh.N[m] * rbits % 128 != 0) return DECDEC_EINVAL;  // a row is a whole number of 16-byte pieces
            bool in_device = false;
            const size_t need = (size_t)sh.K * ((size_t)sh.N[m] * rbits / 8);
            const int prc = check_residual_cached(c.ptrs, lin[m].R_pinned, need, &in_device);
            if (prc != DECDEC_OK) return prc;
            residuals_in_hbm = residuals_in_hbm && in_device;
        }
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const int kind = pack_kind(d0);
    KernelTimer timers[kProfClasses];
    const KernelTimer* tm[kProfClasses] = {nullptr, nullptr, nullptr, nullptr};
    uint8_t* pmask = nullptr;
    if (c.prof_ev != nullptr && c.prof_used < c.prof_cap) {
        hipEvent_t* ev = c.prof_ev + (size_t)c.prof_used * kProfEvents;
        for (int i = 0; i < kProfClasses; ++i) {
            timers[i] = KernelTimer{ev[2 * i], ev[2 * i + 1]};
            tm[i] = &timers[i];
        }
        pmask = c.prof_mask + c.prof_used;
        ++c.prof_used;
    }

    // Split of the work, known up front because every producer must know how many
    // producers a column has in all.
    long tiles = 0;
    for (int m = 0; m < count; ++m) tiles += sh.N[m] / kTileCols;
    // The one-grid kernel is built for fp16 and 4-bit residuals; the other formats take the separate kernels.
    const bool fused = k > 0 && c.mode == DECDEC_MODE_FUSED &&
                       (d0->rfmt == DECDEC_R_FP16 || d0->rfmt == DECDEC_R_INT4_SYM_COL);
    const GemvPlan gp = gemv_plan(tiles, sh.K / kGroup, c.gemv_gpw, fused ? kWavesPerBlock : c.gemv_wpb);
    const int gpw = gp.gpw, wpb = gp.wpb, gslices = gp.slices;
    FetchPlan plan{0, 0, 0};
    if (k > 0) plan = fetch_plan(d0->rfmt, sh, k, c.fetch_split, residuals_in_hbm);
    const int cslices = plan.slices;

    FinalizeArgs fa{};
    for (int m = 0; m < count; ++m) {
        fa.y[m] = static_cast<_Float16*>(ys[m]);
        fa.col0[m] = sh.col0[m];
    }
    fa.acc = c.inkernel_accumulate ? c.acc : nullptr;
    fa.gpart = c.gpart;
    fa.cpart = c.cpart;
    fa.gslices = gslices;
    fa.cslices = cslices;
    fa.Ntot = sh.col0[count];
    // One slice and no residual term: the base GEMV rounds and writes y itself, nothing is left to add.
    fa.direct = k == 0 && gslices == 1 ? 1 : 0;

    if (c.acc_dirty) {
        DD_HIP(launch_clear_u32(reinterpret_cast<unsigned*>(c.acc), 2 * c.maxN, stream));
        c.acc_dirty = 0;
    }
    bool forked = false;  // TWO_STREAMS: the side stream has been made to wait for `stream` and not yet joined back
    const int rc_enq = [&]() -> int {
        if (k == 0) {
            DD_HIP(launch_gemv(kind, sh, gop, x, c.gpart, gslices, gpw, wpb, fa, stream, tm[0]));
            if (pmask) *pmask |= 1;
        } else {
            // The kernels that follow read idx / xsel only; the const is dropped for the shared signatures.
            int32_t* idx = const_cast<int32_t*>(idx_in);
            void* xsel = const_cast<void*>(xsel_in);
            int select_chunks = 0;
            const bool two_streams = c.mode == DECDEC_MODE_TWO_STREAMS;
            hipStream_t comp = two_streams ? c.side : stream;  // where steps 1-3 run
            if (two_streams) {
                // Section 4.1 as printed: compensation on another stream than the base GEMV.
                DD_HIP(hipEventRecord(c.ev_fork, stream));
                DD_HIP(hipStreamWaitEvent(c.side, c.ev_fork, 0));
                forked = true;
            }
            if (!have_idx) {
                idx = c.idx;
                xsel = c.xsel;
                select_chunks = c.separate_select ? 0 : fetch_select_chunks(sh.K, k);
                if (select_chunks == 0) {
                    DD_HIP(launch_select_topk(x, sh.K, k, c.idx, c.xsel, comp, tm[1]));
                    if (pmask) *pmask |= 2;
                }
            }
            if (fused) {
                DD_HIP(launch_compensated_gemv(kind, d0->rfmt, sh, gop, fop, x, select_chunks, idx, xsel, k, c.gpart,
                                               gslices, gpw, c.cpart, plan, fa, stream, tm[2]));
                if (pmask) *pmask |= 4;
            } else {
                DD_HIP(launch_fetch(d0->rfmt, sh, fop, x, select_chunks, idx, xsel, k, c.cpart, plan, fa, comp,
                                    tm[2]));
                if (pmask) *pmask |= 4;
                if (two_streams) DD_HIP(hipEventRecord(c.ev_join, c.side));
                DD_HIP(launch_gemv(kind, sh, gop, x, c.gpart, gslices, gpw, wpb, fa, stream, tm[0]));
                if (pmask) *pmask |= 1;
                if (two_streams) {
                    DD_HIP(hipStreamWaitEvent(stream, c.ev_join, 0));
                    forked = false;
                }
            }
        }
        if (!c.inkernel_accumulate && !fa.direct) {
            DD_HIP(launch_accumulate(sh, ys, c.gpart, gslices, c.cpart, cslices, stream, tm[3]));
            if (pmask) *pmask |= 8;
        }
        return DECDEC_OK;
    }();
    if (rc_enq != DECDEC_OK) {
        c.acc_dirty = 1;  // some producers may never arrive
        if (forked) {
            // Join the side stream back so that `stream` (and a capture in progress) is left whole.
            if (hipEventRecord(c.ev_join, c.side) == hipSuccess) (void)hipStreamWaitEvent(stream, c.ev_join, 0);
            (void)hipGetLastError();
        }
    }
    return rc_enq;
}

decdec_linear one_linear(const decdec_desc* d, const void* Wq, const void* scales, const void* zl, const void* R,
                         const void* Rs, void* y) {
    decdec_linear L;
    L.desc = d;
    L.Wq_dev = Wq;
    L.scales_f16_dev = scales;
    L.zeros_or_lut_f16_dev = zl;
    L.R_pinned = R;
    L.R_scales_f16_dev = Rs;
    L.y_f16_dev = y;
    return L;
}

}  // namespace

extern "C" {

int decdec_gemv(const decdec_desc* d, const void* x_f16_dev, const void* Wq_dev, const void* scales_f16_dev,
                const void* zeros_or_lut_f16_dev, const void* R_pinned, const void* R_scales_f16_dev, int32_t k,
                void* y_f16_dev, decdec_ws* ws, void* stream) {
    if (d == nullptr || ws == nullptr) return DECDEC_EINVAL;
    const decdec_linear L =
        one_linear(d, Wq_dev, scales_f16_dev, zeros_or_lut_f16_dev, R_pinned, R_scales_f16_dev, y_f16_dev);
    return gemv_common(1, &L, x_f16_dev, k, nullptr, nullptr, false, &ws->core, stream);
}

int decdec_gemv_idx(const decdec_desc* d, const void* x_f16_dev, const void* Wq_dev, const void* scales_f16_dev,
                    const void* zeros_or_lut_f16_dev, const void* R_pinned, const void* R_scales_f16_dev, int32_t k,
                    const int32_t* idx_dev, const void* xsel_f16_dev, void* y_f16_dev, decdec_ws* ws, void* stream) {
    if (d == nullptr || ws == nullptr) return DECDEC_EINVAL;
    const decdec_linear L =
        one_linear(d, Wq_dev, scales_f16_dev, zeros_or_lut_f16_dev, R_pinned, R_scales_f16_dev, y_f16_dev);
    return gemv_common(1, &L, x_f16_dev, k, idx_dev, xsel_f16_dev, true, &ws->core, stream);
}

int decdec_gemv_multi(int32_t count, const decdec_linear* linears, const void* x_f16_dev, int32_t k, decdec_ws* ws,
                      void* stream) {
    if (ws == nullptr) return DECDEC_EINVAL;
    return gemv_common(count, linears, x_f16_dev, k, nullptr, nullptr, false, &ws->core, stream);
}

// ------------------------------------------------ the entry point that allocates nothing

}  // extern "C"

namespace {

constexpr size_t round256(size_t n) { return (n + 255) / 256 * 256; }
constexpr size_t kStIdxOff = 0;
constexpr size_t kStXselOff = kStIdxOff + round256((size_t)DECDEC_STATIC_MAX_SELECTED * 4);
constexpr size_t kStAccOff = kStXselOff + round256((size_t)DECDEC_STATIC_MAX_SELECTED * 2);
constexpr size_t kStaticScratchBytes = kStAccOff + (size_t)DECDEC_STATIC_MAX_N * 8;

constexpr int kMaxDevices = 16;
struct StaticState {
    Core core;  // buffers point into this GPU's copy of `scratch`
    PtrEntry slots[kStaticPointerSlots];
    bool ready;
};
StaticState g_static[kMaxDevices];  // zero-initialised; entry d belongs to GPU d
std::mutex g_static_mutex;

}  // namespace

// Scratch memory of decdec_gemv_static: the selection buffer and the per-column accumulators the producers
// add into, for problems up to DECDEC_STATIC_MAX_N columns and DECDEC_STATIC_MAX_SELECTED channels.
// Every GPU the library runs on holds its own copy at its own address until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; kernels receive the address that call returns.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

extern "C" {

int decdec_gemv_static(const decdec_desc* d, const void* x_f16_dev, const void* Wq_dev, const void* scales_f16_dev,
                       const void* zeros_or_lut_f16_dev, const void* R_pinned, const void* R_scales_f16_dev,
                       int32_t k, void* y_f16_dev, void* stream) {
    if (d == nullptr) return DECDEC_EINVAL;
    int dev = -1;
    DD_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return DECDEC_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticState& st = g_static[dev];
    if (!st.ready) {
        // Once per GPU, with that GPU current: the address of its copy of the array.
        void* ptr = nullptr;
        DD_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (ptr == nullptr) return hip_fail(hipErrorInvalidSymbol);
        unsigned char* base = static_cast<unsigned char*>(ptr);
        Core& c = st.core;
        std::memset(&c, 0, sizeof(c));
        c.maxK = kSelectMaxK;
        c.maxN = DECDEC_STATIC_MAX_N;
        c.maxk = DECDEC_STATIC_MAX_SELECTED;
        c.idx = reinterpret_cast<int32_t*>(base + kStIdxOff);
        c.xsel = base + kStXselOff;
        c.acc = reinterpret_cast<unsigned long long*>(base + kStAccOff);
        c.ptrs.e = st.slots;
        c.ptrs.cap = kStaticPointerSlots;
        c.inkernel_accumulate = 1;
        c.acc_dirty = 1;  // the first call clears the accumulators with a fill kernel on its stream
        st.ready = true;
    }
    if (check_desc(d) == DECDEC_OK && (d->N > DECDEC_STATIC_MAX_N || k > DECDEC_STATIC_MAX_SELECTED))
        return DECDEC_ETOOLARGE;
    const decdec_linear L =
        one_linear(d, Wq_dev, scales_f16_dev, zeros_or_lut_f16_dev, R_pinned, R_scales_f16_dev, y_f16_dev);
    return gemv_common(1, &L, x_f16_dev, k, nullptr, nullptr, false, &st.core, stream);
}

// ------------------------------------------------ offline, on the device

int decdec_quantize_uniform(const decdec_desc* d, const void* W_f32_dev, void* Wq_out_dev, void* scales_f16_out_dev,
                            void* zeros_f16_out_dev, void* R_f16_out, void* stream) {
    const int rc = check_desc(d);
    if (rc != DECDEC_OK) return rc;
    if (d->wfmt != DECDEC_W_UNIFORM_G128) return DECDEC_EUNSUPPORTED;
    if (W_f32_dev == nullptr || Wq_out_dev == nullptr || scales_f16_out_dev == nullptr ||
        zeros_f16_out_dev == nullptr)
        return DECDEC_EINVAL;
    DD_HIP(launch_quantize_uniform(d->wbits, static_cast<const float*>(W_f32_dev), Wq_out_dev, scales_f16_out_dev,
                                   zeros_f16_out_dev, R_f16_out, d->K, d->N, static_cast<hipStream_t>(stream)));
    return DECDEC_OK;
}

int decdec_residual_f32(const decdec_desc* d, const void* W_f32_dev, const void* Wq_dev, const void* scales_f16_dev,
                        const void* zeros_or_lut_f16_dev, void* R_f32_out_dev, void* stream) {
    const int rc = check_desc(d);
    if (rc != DECDEC_OK) return rc;
    if (W_f32_dev == nullptr || Wq_dev == nullptr || zeros_or_lut_f16_dev == nullptr || R_f32_out_dev == nullptr)
        return DECDEC_EINVAL;
    if (d->wfmt == DECDEC_W_UNIFORM_G128 && scales_f16_dev == nullptr) return DECDEC_EINVAL;
    DD_HIP(launch_residual_f32(pack_kind(d), static_cast<const float*>(W_f32_dev), Wq_dev, scales_f16_dev,
                               zeros_or_lut_f16_dev, static_cast<float*>(R_f32_out_dev), d->K, d->N,
                               static_cast<hipStream_t>(stream)));
    return DECDEC_OK;
}

int decdec_quantize_residual(int32_t K, int32_t N, int32_t bits, const void* R_f32_dev, void* codes_out,
                             void* scales_f16_out_dev, void* stream) {
    if (bits != 2 && bits != 4 && bits != 8) return DECDEC_EUNSUPPORTED;
    if (K <= 0 || N <= 0 || N % (128 / bits) != 0 || R_f32_dev == nullptr || codes_out == nullptr ||
        scales_f16_out_dev == nullptr)
        return DECDEC_EINVAL;
    DD_HIP(launch_quantize_residual(bits, static_cast<const float*>(R_f32_dev), codes_out, scales_f16_out_dev, K, N,
                                    static_cast<hipStream_t>(stream)));
    return DECDEC_OK;
}

}  // extern "C"
