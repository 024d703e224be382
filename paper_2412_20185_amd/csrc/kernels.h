// Internal launch interface between the C-ABI layer (api.hip) and the kernel
// translation units.  Every launcher validates nothing: api.hip has already
// checked shapes against what the kernels and their grids assume.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace decdec {

constexpr int kMaxGemvSlices = 64;   // fp32 partial rows the base GEMV may write
constexpr int kMaxFetchSlices = 64;  // fp32 partial rows the residual kernel may write
constexpr int kSelectThreads = 1024;
constexpr int kSelectMaxK = 65536;

// gemv.hip ---------------------------------------------------------------
// part: fp32 [slices][N]; *slices_out receives the number of rows written.
hipError_t launch_gemv(int kind, const void* Wq, const void* scales, const void* zeros_or_lut, const void* x,
                       float* part, int K, int N, int gpw_request, int* slices_out, hipStream_t stream);
int gemv_slices(int N, int G, int gpw_request, int* gpw_out);

// select.hip -------------------------------------------------------------
hipError_t launch_select_topk(const void* x, int K, int k, int32_t* idx_out, void* xsel_out, hipStream_t stream);

// fetch.hip --------------------------------------------------------------
// cpart: fp32 [slices][N]; row_split: requested slices (0 = automatic).
int fetch_slices(int rfmt, int N, int k, int row_split);
hipError_t launch_fetch(int rfmt, const void* R_pinned, const void* R_scales, const int32_t* idx, const void* xsel,
                        int k, int K, int N, float* cpart, int slices, hipStream_t stream);

// accumulate.hip ---------------------------------------------------------
// y[n] = fp16( sum_s gpart[s][n] + sum_r cpart[r][n] )
hipError_t launch_accumulate(const float* gpart, int gslices, const float* cpart, int cslices, int N, void* y,
                             hipStream_t stream);

// quantize.hip -----------------------------------------------------------
hipError_t launch_quantize_uniform(int bits, const float* W, void* Wq, void* scales, void* zeros, void* R, int K,
                                   int N, hipStream_t stream);

}  // namespace decdec
