// C ABI of the library (see include/decdec.h): argument checking, the host
// helpers that convert plain code matrices to the private packed layout, and
// the stream choreography of one compensated GEMV.
#include <hip/hip_runtime.h>

#include <cstring>
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

constexpr int kPinnedCache = 16;
constexpr int kProfClasses = 4;              // base GEMV, selection, fetch, accumulate
constexpr int kProfEvents = 2 * kProfClasses;  // a (start, stop) pair each

}  // namespace

struct decdec_ws {
    int32_t maxK, maxN, maxk;
    int32_t fetch_split;
    int32_t gemv_gpw;
    hipStream_t side;
    hipEvent_t ev_fork, ev_join;
    int32_t* idx;    // [maxk]
    void* xsel;      // fp16 [maxk]
    float* gpart;    // [kMaxGemvSlices][maxN]
    float* cpart;    // [kMaxFetchSlices][maxN]
    unsigned* counters;  // [maxN/64] per-tile arrival counters, zero between calls
    int32_t mode;                 // decdec_mode
    int32_t separate_select;      // 1: selection always runs as a kernel of its own
    int32_t inkernel_accumulate;  // 1: the last producer of a tile adds the partial rows (no accumulate kernel)
    int32_t counters_dirty;       // a call failed half-way: clear the counters before the next one
    const void* pinned_ok[kPinnedCache];  // residual base pointers already verified
    uint8_t pinned_dev[kPinnedCache];     // 1: that pointer is device memory
    int pinned_n, pinned_next;
    // optional kernel timing: per call one (start, stop) event pair per kernel class
    hipEvent_t* prof_ev;   // [prof_cap][kProfEvents]: gemv, select, fetch, accumulate
    uint8_t* prof_mask;    // [prof_cap] bit c: class c was launched and timed
    int32_t prof_cap, prof_used;
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
        default: return "unknown status";
    }
}

int decdec_last_hip_error(void) { return g_last_hip_error; }

size_t decdec_sc_buffer_bytes(int32_t k) { return k > 0 ? (size_t)k * (4 + 2) : 0; }

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
    ws->maxK = maxK;
    ws->maxN = maxN;
    ws->maxk = maxk;
    const size_t kk = maxk > 0 ? (size_t)maxk : 1;
    hipError_t e = hipStreamCreateWithFlags(&ws->side, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ws->ev_fork, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ws->ev_join, hipEventDisableTiming);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ws->idx), kk * 4);
    if (e == hipSuccess) e = hipMalloc(&ws->xsel, kk * 2);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ws->gpart), (size_t)kMaxGemvSlices * maxN * 4);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ws->cpart), (size_t)kMaxFetchSlices * maxN * 4);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ws->counters), ((size_t)maxN / 64 + 1) * 4);
    if (e == hipSuccess) e = hipMemset(ws->counters, 0, ((size_t)maxN / 64 + 1) * 4);
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

static void free_profiling(decdec_ws* ws) {
    if (ws->prof_ev) {
        for (int i = 0; i < ws->prof_cap * kProfEvents; ++i)
            if (ws->prof_ev[i]) (void)hipEventDestroy(ws->prof_ev[i]);
        delete[] ws->prof_ev;
        delete[] ws->prof_mask;
    }
    ws->prof_ev = nullptr;
    ws->prof_mask = nullptr;
    ws->prof_cap = ws->prof_used = 0;
}

int decdec_ws_set_profiling(decdec_ws* ws, int32_t capacity) {
    if (ws == nullptr || capacity < 0 || capacity > (1 << 20)) return DECDEC_EINVAL;
    DD_HIP(hipDeviceSynchronize());
    free_profiling(ws);
    if (capacity == 0) return DECDEC_OK;
    ws->prof_ev = new (std::nothrow) hipEvent_t[(size_t)capacity * kProfEvents]();
    ws->prof_mask = new (std::nothrow) uint8_t[capacity]();
    if (ws->prof_ev == nullptr || ws->prof_mask == nullptr) {
        delete[] ws->prof_ev;
        delete[] ws->prof_mask;
        ws->prof_ev = nullptr;
        ws->prof_mask = nullptr;
        return DECDEC_ENOMEM;
    }
    ws->prof_cap = capacity;
    for (int i = 0; i < capacity * kProfEvents; ++i) {
        const hipError_t e = hipEventCreate(&ws->prof_ev[i]);
        if (e != hipSuccess) {
            free_profiling(ws);
            return hip_fail(e);
        }
    }
    return DECDEC_OK;
}

int decdec_ws_read_profile(decdec_ws* ws, double* ms_out, int32_t* calls_out) {
    if (ws == nullptr) return DECDEC_EINVAL;
    double t[kProfClasses] = {0, 0, 0, 0};
    int32_t n[kProfClasses] = {0, 0, 0, 0};
    if (ws->prof_ev) {
        DD_HIP(hipDeviceSynchronize());
        for (int i = 0; i < ws->prof_used; ++i) {
            hipEvent_t* ev = ws->prof_ev + (size_t)i * kProfEvents;
            for (int c = 0; c < kProfClasses; ++c) {
                if (ws->prof_mask[i] & (1 << c)) {
                    float ms = 0.f;
                    DD_HIP(hipEventElapsedTime(&ms, ev[2 * c], ev[2 * c + 1]));
                    t[c] += ms;
                    ++n[c];
                }
            }
            ws->prof_mask[i] = 0;
        }
        ws->prof_used = 0;
    }
    for (int c = 0; c < kProfClasses; ++c) {
        if (ms_out) ms_out[c] = t[c];
        if (calls_out) calls_out[c] = n[c];
    }
    return DECDEC_OK;
}

int decdec_ws_destroy(decdec_ws* ws) {
    if (ws == nullptr) return DECDEC_OK;
    free_profiling(ws);
    if (ws->side) {
        (void)hipStreamSynchronize(ws->side);
        (void)hipStreamDestroy(ws->side);
    }
    if (ws->ev_fork) (void)hipEventDestroy(ws->ev_fork);
    if (ws->ev_join) (void)hipEventDestroy(ws->ev_join);
    if (ws->idx) (void)hipFree(ws->idx);
    if (ws->xsel) (void)hipFree(ws->xsel);
    if (ws->gpart) (void)hipFree(ws->gpart);
    if (ws->cpart) (void)hipFree(ws->cpart);
    if (ws->counters) (void)hipFree(ws->counters);
    delete ws;
    return DECDEC_OK;
}

int decdec_ws_last_selection(const decdec_ws* ws, const int32_t** idx_dev, const void** xsel_f16_dev) {
    if (ws == nullptr) return DECDEC_EINVAL;
    if (idx_dev) *idx_dev = ws->idx;
    if (xsel_f16_dev) *xsel_f16_dev = ws->xsel;
    return DECDEC_OK;
}

int decdec_ws_set_inkernel_accumulate(decdec_ws* ws, int32_t on) {
    if (ws == nullptr || (on != 0 && on != 1)) return DECDEC_EINVAL;
    ws->inkernel_accumulate = on;
    return DECDEC_OK;
}

int decdec_ws_set_mode(decdec_ws* ws, int32_t mode) {
    if (ws == nullptr || mode < DECDEC_MODE_FUSED || mode > DECDEC_MODE_TWO_STREAMS) return DECDEC_EINVAL;
    ws->mode = mode;
    return DECDEC_OK;
}

int decdec_ws_set_separate_select(decdec_ws* ws, int32_t on) {
    if (ws == nullptr || (on != 0 && on != 1)) return DECDEC_EINVAL;
    ws->separate_select = on;
    return DECDEC_OK;
}

int decdec_ws_set_gemv_split(decdec_ws* ws, int32_t groups_per_wave) {
    if (ws == nullptr || groups_per_wave < 0 || groups_per_wave > 1024) return DECDEC_EINVAL;
    ws->gemv_gpw = groups_per_wave;
    return DECDEC_OK;
}

int decdec_ws_read_selection(const decdec_ws* ws, int32_t k, int32_t* idx_host, void* xsel_f16_host) {
    if (ws == nullptr || k < 0 || k > ws->maxk) return DECDEC_EINVAL;
    DD_HIP(hipStreamSynchronize(ws->side));
    if (k == 0) return DECDEC_OK;
    if (idx_host) DD_HIP(hipMemcpy(idx_host, ws->idx, (size_t)k * 4, hipMemcpyDeviceToHost));
    if (xsel_f16_host) DD_HIP(hipMemcpy(xsel_f16_host, ws->xsel, (size_t)k * 2, hipMemcpyDeviceToHost));
    return DECDEC_OK;
}

int decdec_ws_set_fetch_split(decdec_ws* ws, int32_t row_split) {
    if (ws == nullptr || row_split < 0 || row_split > kMaxFetchSlices) return DECDEC_EINVAL;
    ws->fetch_split = row_split;
    return DECDEC_OK;
}

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
    if (k == 0) return DECDEC_OK;
    if (idx_out_dev == nullptr) return DECDEC_EINVAL;
    DD_HIP(launch_select_topk(x_f16_dev, K, k, idx_out_dev, xsel_f16_dev, static_cast<hipStream_t>(stream)));
    return DECDEC_OK;
}

int decdec_select_bucket(const void* x_f16_dev, int32_t K, int32_t k_chunk, float b0, float b15,
                         int32_t* idx_out_dev, void* xsel_f16_dev, void* stream) {
    if (x_f16_dev == nullptr || K < 1024 || K % 1024 != 0 || k_chunk < 0 || k_chunk > 1024) return DECDEC_EINVAL;
    if (!(b0 >= b15) || !(b15 >= 0.f)) return DECDEC_EINVAL;  // also rejects NaN
    if (k_chunk == 0) return DECDEC_OK;
    if (idx_out_dev == nullptr) return DECDEC_EINVAL;
    DD_HIP(launch_select_bucket(x_f16_dev, K, k_chunk, b0, b15, idx_out_dev, xsel_f16_dev,
                                static_cast<hipStream_t>(stream)));
    return DECDEC_OK;
}

// *in_device: the residuals live in device memory (not over the host link).
static int check_pinned_cached(decdec_ws* ws, const void* R_pinned, bool* in_device) {
    for (int i = 0; i < ws->pinned_n; ++i) {
        if (ws->pinned_ok[i] == R_pinned) {
            *in_device = ws->pinned_dev[i] != 0;
            return DECDEC_OK;
        }
    }
    const int type = residual_memory_type(R_pinned);
    if (type < 0) return DECDEC_ENOTPINNED;
    *in_device = type == (int)hipMemoryTypeDevice;
    ws->pinned_ok[ws->pinned_next] = R_pinned;
    ws->pinned_dev[ws->pinned_next] = *in_device ? 1 : 0;
    ws->pinned_next = (ws->pinned_next + 1) % kPinnedCache;
    if (ws->pinned_n < kPinnedCache) ++ws->pinned_n;
    return DECDEC_OK;
}

// count linears that share x (and therefore K, the selection, and one launch
// of each kernel).  idx_in/xsel_in: caller-supplied selection or null.
static int gemv_common(int32_t count, const decdec_linear* lin, const void* x, int32_t k, const int32_t* idx_in,
                       const void* xsel_in, bool have_idx, decdec_ws* ws, void* stream_v) {
    if (lin == nullptr || count < 1 || count > kMaxMulti || ws == nullptr || x == nullptr) return DECDEC_EINVAL;
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
    if (sh.K > ws->maxK || sh.col0[count] > ws->maxN || k < 0 || k > sh.K || k > ws->maxk) return DECDEC_EINVAL;
    bool residuals_in_hbm = k > 0;  // all of them: the fetch is then bound by HBM latency, not by the host link
    if (k > 0) {
        if (have_idx && (idx_in == nullptr || xsel_in == nullptr)) return DECDEC_EINVAL;
        for (int m = 0; m < count; ++m) {
            if (lin[m].R_pinned == nullptr) return DECDEC_EINVAL;
            if (d0->rfmt != DECDEC_R_FP16 && lin[m].R_scales_f16_dev == nullptr) return DECDEC_EINVAL;
            bool in_device = false;
            const int prc = check_pinned_cached(ws, lin[m].R_pinned, &in_device);
            if (prc != DECDEC_OK) return prc;
            residuals_in_hbm = residuals_in_hbm && in_device;
        }
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const int kind = pack_kind(d0);
    KernelTimer timers[kProfClasses];
    const KernelTimer* tm[kProfClasses] = {nullptr, nullptr, nullptr, nullptr};
    uint8_t* pmask = nullptr;
    if (ws->prof_ev != nullptr && ws->prof_used < ws->prof_cap) {
        hipEvent_t* ev = ws->prof_ev + (size_t)ws->prof_used * kProfEvents;
        for (int c = 0; c < kProfClasses; ++c) {
            timers[c] = KernelTimer{ev[2 * c], ev[2 * c + 1]};
            tm[c] = &timers[c];
        }
        pmask = ws->prof_mask + ws->prof_used;
        ++ws->prof_used;
    }

    // Split of the work, known up front because each kernel must know how many
    // partial rows the other one contributes.
    long tiles = 0;
    for (int m = 0; m < count; ++m) tiles += sh.N[m] / kTileCols;
    // The one-grid kernel is built for fp16 and 4-bit residuals; the other formats take the separate kernels.
    const bool fused = k > 0 && ws->mode == DECDEC_MODE_FUSED &&
                       (d0->rfmt == DECDEC_R_FP16 || d0->rfmt == DECDEC_R_INT4_SYM_COL);
    int gpw = 1;
    const int gslices =
        gemv_slices(tiles, sh.K / kGroup, ws->gemv_gpw, fused ? kWavesPerBlock : kGemvAloneWaves, &gpw);
    const int cslices = k > 0 ? fetch_slices(d0->rfmt, sh, k, ws->fetch_split, residuals_in_hbm) : 0;

    FinalizeArgs fa{};
    int t0 = 0;
    for (int m = 0; m < count; ++m) {
        fa.y[m] = static_cast<_Float16*>(ys[m]);
        fa.col0[m] = sh.col0[m];
        fa.tile0[m] = t0;
        t0 += sh.N[m] / kTileCols;
    }
    fa.gpart = ws->gpart;
    fa.cpart = ws->cpart;
    fa.gslices = gslices;
    fa.cslices = cslices;
    fa.Ntot = sh.col0[count];
    fa.counters = ws->inkernel_accumulate ? ws->counters : nullptr;

    if (ws->counters_dirty) {
        DD_HIP(launch_clear_u32(ws->counters, ws->maxN / 64 + 1, stream));
        ws->counters_dirty = 0;
    }
    const int rc_enq = [&]() -> int {
        if (k == 0) {
            DD_HIP(launch_gemv(kind, sh, gop, x, ws->gpart, gslices, gpw, fa, stream, tm[0]));
            if (pmask) *pmask |= 1;
        } else {
            // The kernels that follow read idx / xsel only; the const is dropped for the shared signatures.
            int32_t* idx = const_cast<int32_t*>(idx_in);
            void* xsel = const_cast<void*>(xsel_in);
            int select_chunks = 0;
            const bool two_streams = ws->mode == DECDEC_MODE_TWO_STREAMS;
            hipStream_t comp = two_streams ? ws->side : stream;  // where steps 1-3 run
            if (two_streams) {
                // Section 4.1 as printed: compensation on another stream than the base GEMV.
                DD_HIP(hipEventRecord(ws->ev_fork, stream));
                DD_HIP(hipStreamWaitEvent(ws->side, ws->ev_fork, 0));
            }
            if (!have_idx) {
                idx = ws->idx;
                xsel = ws->xsel;
                select_chunks = ws->separate_select ? 0 : fetch_select_chunks(sh.K, k);
                if (select_chunks == 0) {
                    DD_HIP(launch_select_topk(x, sh.K, k, ws->idx, ws->xsel, comp, tm[1]));
                    if (pmask) *pmask |= 2;
                }
            }
            if (fused) {
                DD_HIP(launch_compensated_gemv(kind, d0->rfmt, sh, gop, fop, x, select_chunks, idx, xsel, k, ws->gpart,
                                               gslices, gpw, ws->cpart, cslices, fa, stream, tm[2]));
                if (pmask) *pmask |= 4;
            } else {
                DD_HIP(launch_fetch(d0->rfmt, sh, fop, x, select_chunks, idx, xsel, k, ws->cpart, cslices, fa, comp,
                                    tm[2]));
                if (pmask) *pmask |= 4;
                if (two_streams) DD_HIP(hipEventRecord(ws->ev_join, ws->side));
                DD_HIP(launch_gemv(kind, sh, gop, x, ws->gpart, gslices, gpw, fa, stream, tm[0]));
                if (pmask) *pmask |= 1;
                if (two_streams) DD_HIP(hipStreamWaitEvent(stream, ws->ev_join, 0));
            }
        }
        if (!ws->inkernel_accumulate) {
            DD_HIP(launch_accumulate(sh, ys, ws->gpart, gslices, ws->cpart, cslices, stream, tm[3]));
            if (pmask) *pmask |= 8;
        }
        return DECDEC_OK;
    }();
    if (rc_enq != DECDEC_OK) ws->counters_dirty = 1;  // some producers may never arrive
    return rc_enq;
}

static decdec_linear one_linear(const decdec_desc* d, const void* Wq, const void* scales, const void* zl,
                                const void* R, const void* Rs, void* y) {
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

int decdec_gemv(const decdec_desc* d, const void* x_f16_dev, const void* Wq_dev, const void* scales_f16_dev,
                const void* zeros_or_lut_f16_dev, const void* R_pinned, const void* R_scales_f16_dev, int32_t k,
                void* y_f16_dev, decdec_ws* ws, void* stream) {
    if (d == nullptr) return DECDEC_EINVAL;
    const decdec_linear L =
        one_linear(d, Wq_dev, scales_f16_dev, zeros_or_lut_f16_dev, R_pinned, R_scales_f16_dev, y_f16_dev);
    return gemv_common(1, &L, x_f16_dev, k, nullptr, nullptr, false, ws, stream);
}

int decdec_gemv_idx(const decdec_desc* d, const void* x_f16_dev, const void* Wq_dev, const void* scales_f16_dev,
                    const void* zeros_or_lut_f16_dev, const void* R_pinned, const void* R_scales_f16_dev, int32_t k,
                    const int32_t* idx_dev, const void* xsel_f16_dev, void* y_f16_dev, decdec_ws* ws, void* stream) {
    if (d == nullptr) return DECDEC_EINVAL;
    const decdec_linear L =
        one_linear(d, Wq_dev, scales_f16_dev, zeros_or_lut_f16_dev, R_pinned, R_scales_f16_dev, y_f16_dev);
    return gemv_common(1, &L, x_f16_dev, k, idx_dev, xsel_f16_dev, true, ws, stream);
}

int decdec_gemv_multi(int32_t count, const decdec_linear* linears, const void* x_f16_dev, int32_t k, decdec_ws* ws,
                      void* stream) {
    return gemv_common(count, linears, x_f16_dev, k, nullptr, nullptr, false, ws, stream);
}

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
