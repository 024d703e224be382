// Internal launch interface between the C-ABI layer (api.hip) and the kernel
// translation units.  Every launcher validates nothing: api.hip has already
// checked shapes against what the kernels and their grids assume.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <cstdint>

namespace decdec {

// Workgroup size of the base-GEMV, residual and fused kernels (one wavefront = one unit of work in all of them).
constexpr int kBlockThreads = 512;
constexpr int kWavesPerBlock = kBlockThreads / 64;

constexpr int kMaxGemvSlices = 16;   // part sums per column the base GEMV may contribute (K-slices)
constexpr int kMaxFetchSlices = 16;  // part sums per column the residual kernel may contribute (row slices)
constexpr int kSelectThreads = 1024;
constexpr int kSelectMaxK = 65536;

// Optional pair of events that receive the begin and end timestamps of one
// kernel dispatch (what a kernel trace reports as its duration).
struct KernelTimer {
    hipEvent_t start, stop;
};

// Launches `kernel`; with a timer the dispatch's own timestamps go to its events.
template <typename F, typename... Args>
inline hipError_t launch_kernel(const KernelTimer* tm, F kernel, dim3 grid, dim3 block, unsigned lds,
                                hipStream_t stream, Args... args) {
    if (tm != nullptr) {
        hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, tm->start, tm->stop, 0, args...);
    } else {
        kernel<<<grid, block, lds, stream>>>(args...);
    }
    return hipGetLastError();
}

// One call handles up to kMaxMulti weight matrices that share the activation
// vector x (q/k/v, gate/up): their columns are treated as one concatenated
// output of Ntot = sum N_m columns; matrix m owns columns [col0[m], col0[m]+N[m]).
constexpr int kMaxMulti = 4;

struct MultiShape {
    int n;                    // matrices in this call
    int K;                    // shared input channels
    int N[kMaxMulti];         // output columns per matrix
    int col0[kMaxMulti + 1];  // first concatenated column of matrix m; col0[n] = Ntot
};

struct GemvOperands {
    const void* Wq[kMaxMulti];
    const void* scales[kMaxMulti];
    const void* zeros_or_lut[kMaxMulti];
};

struct FetchOperands {
    const void* R[kMaxMulti];         // pinned residual rows
    const void* R_scales[kMaxMulti];  // fp16 [N_m] (int4 residuals) or null
};

// gemv.hip ---------------------------------------------------------------
// part: fp32 [slices][Ntot], written only when fa.acc is null (a separate kernel adds the rows); may be null otherwise.
struct FinalizeArgs;
// wpb: wavefronts per workgroup (4, 8 or 16).
hipError_t launch_gemv(int kind, const MultiShape& sh, const GemvOperands& op, const void* x, float* part,
                       int slices, int gpw, int wpb, const FinalizeArgs& fa, hipStream_t stream,
                       const KernelTimer* tm = nullptr);
// How K is cut: workgroups of `wpb` wavefronts, each wavefront walking `gpw` groups of 128 input channels,
// `slices` workgroups (and part sums per column) per 64-column tile.  Requests of 0 leave the choice to the
// library; inside the one-grid kernel wpb is kWavesPerBlock.
struct GemvPlan {
    int wpb, gpw, slices;
};
GemvPlan gemv_plan(long tiles, int G, int gpw_request, int wpb_request);

// select.hip -------------------------------------------------------------
hipError_t launch_select_topk(const void* x, int K, int k, int32_t* idx_out, void* xsel_out, hipStream_t stream,
                              const KernelTimer* tm = nullptr);

// select_bucket.hip ------------------------------------------------------
// The paper's approximate Top-K: k_chunk channels per 1024-channel chunk (K a multiple of 1024).
hipError_t launch_select_bucket(const void* x, int K, int k_chunk, float b0, float b15, int32_t* idx_out,
                                void* xsel_out, hipStream_t stream, const KernelTimer* tm = nullptr);

// fetch.hip --------------------------------------------------------------
// How the residual kernel is laid out: `segments` column segments (one 16-byte piece per lane and row; all
// matrices of the call together) x `slices` workgroups per segment; `row_waves` wavefronts of each workgroup
// share its rows.  cpart is fp32 [slices][Ntot] (used only when fa.acc is null).
struct FetchPlan {
    int segments, slices, row_waves;
};
// row_split: requested workgroups per segment (0 = automatic); in_hbm: the residual rows are in device
// memory, not behind the host link.
FetchPlan fetch_plan(int rfmt, const MultiShape& sh, int k, int row_split, bool in_hbm);
// select_chunks (from fetch_select_chunks) > 0: the kernel runs the exact top-k on x itself and writes
// the selection to idx / xsel; 0: idx / xsel hold the selection already (x is not read).
int fetch_select_chunks(int K, int k);
hipError_t launch_fetch(int rfmt, const MultiShape& sh, const FetchOperands& op, const void* x, int select_chunks,
                        int32_t* idx, void* xsel, int k, float* cpart, const FetchPlan& plan, const FinalizeArgs& fa,
                        hipStream_t stream, const KernelTimer* tm = nullptr);

// fused.hip -------------------------------------------------------------
// Base GEMV and residual kernel in one grid (the fetch workgroups come first).
hipError_t launch_compensated_gemv(int kind, int rfmt, const MultiShape& sh, const GemvOperands& gop,
                                   const FetchOperands& fop, const void* x, int select_chunks, int32_t* idx, void* xsel,
                                   int k, float* gpart, int gslices, int gpw, float* cpart, const FetchPlan& plan,
                                   const FinalizeArgs& fa, hipStream_t stream, const KernelTimer* tm = nullptr);

// accumulate.hip ---------------------------------------------------------
// y_m[n] = fp16( sum_s gpart[s][col0[m]+n] + sum_r cpart[r][col0[m]+n] ), the terms added in the fixed point of finalize.h
hipError_t launch_accumulate(const MultiShape& sh, void* const* y, const float* gpart, int gslices,
                             const float* cpart, int cslices, hipStream_t stream, const KernelTimer* tm = nullptr);

// A fill kernel (not hipMemsetAsync, so that callers may capture the call in a graph).
hipError_t launch_clear_u32(unsigned* p, int n, hipStream_t stream);

// quantize.hip -----------------------------------------------------------
hipError_t launch_quantize_uniform(int bits, const float* W, void* Wq, void* scales, void* zeros, void* R, int K,
                                   int N, hipStream_t stream);
hipError_t launch_residual_f32(int kind, const float* W, const void* Wq, const void* scales, const void* zeros_or_lut,
                               float* R, int K, int N, hipStream_t stream);
hipError_t launch_quantize_residual(int bits, const float* R, void* codes_out, void* scales_out, int K, int N,
                                    hipStream_t stream);

}  // namespace decdec
