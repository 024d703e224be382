/*
 * decdec.h - C ABI of the DecDEC decode-step hot path for AMD MI355X (gfx950).
 *
 * One call computes, for one linear layer at batch 1,
 *
 *     o = W_hat x  +  R_hat[sc_indices, :]^T x[sc_indices]
 *
 * where W_hat is the de-quantised 3/4-bit weight matrix resident in GPU
 * memory, R_hat the residual W - W_hat resident in pinned CPU memory (the
 * paper's placement; GPU memory is accepted too), and
 * sc_indices the k input channels with the largest |x| of THIS step
 * (DecDEC, Section 3.1 "(W_hat + R o M) x" and Section 4.1 steps 1-4).
 *
 * Orientation (Section 3.1-3.2, 4.2): a weight matrix is d_in x d_out = K x N;
 * an input channel is a row, an output channel a column.  x has K entries,
 * o has N entries.
 *
 * Conventions
 *   - "dev"  pointer: GPU memory (hipMalloc / a torch CUDA tensor).
 *   - "host" pointer: ordinary CPU memory, touched only by the host helpers.
 *   - "pinned" pointer: page-locked, GPU-mapped CPU memory (hipHostMalloc or
 *     a torch tensor with pin_memory=True); kernels read it in place over the
 *     host link (Section 4.3 "Zero-Copy Residual Fetch").
 *   - fp16 = IEEE binary16.  All multi-dimensional arrays are row-major.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Hot-path calls only enqueue work: no allocation, no host
 *     synchronisation.  When a call returns, `stream` is ordered after the
 *     result.  Pointers are borrowed until that work has run.
 *   - Every function returns a decdec_status (0 = OK, negative = error);
 *     nothing throws, aborts or prints.  A call that fails validation
 *     (EINVAL, EUNSUPPORTED, ENOTPINNED, ETOOLARGE) has enqueued nothing.  A
 *     call that fails with EHIP (a launch was refused) may have enqueued some
 *     of its kernels already: y is then undefined, the stream stays usable
 *     (in TWO_STREAMS mode the second stream has been joined back) and the
 *     workspace cleans up after itself on its next call.
 *   - Alignment: x, Wq, the codebook, residual rows and residual scales are
 *     read with 128-bit loads and must be 16-byte aligned; fp16 arrays that are
 *     read or written element-wise (scales, zero points, y, xsel) 2-byte and
 *     index arrays 4-byte aligned.  Anything else is DECDEC_EINVAL.
 *   - A workspace serialises its users: calls that share one decdec_ws must
 *     be issued on one stream (or otherwise ordered); use one workspace per
 *     concurrent stream.
 */
#ifndef DECDEC_H
#define DECDEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DECDEC_OK = 0,
    DECDEC_EINVAL = -1,       /* null pointer, size or k out of range, bad alignment */
    DECDEC_EUNSUPPORTED = -2, /* format / bit-width combination not implemented */
    DECDEC_ENOTPINNED = -3,   /* residual pointer is neither pinned host memory nor device memory */
    DECDEC_EHIP = -4,         /* a HIP runtime call failed; see decdec_last_hip_error */
    DECDEC_ENOMEM = -5,       /* workspace allocation failed */
    DECDEC_ETOOLARGE = -6     /* decdec_gemv_static: N or k beyond what its fixed scratch buffer holds */
} decdec_status;

/* Base-weight formats (what the base GEMV de-quantises).
 *   UNIFORM_G128: b-bit codes, b in {3,4}; W_hat[k][n] = s[k/128][n] * (q[k][n] - z[k/128][n])
 *                 with fp16 scale s and integer-valued fp16 zero point z per
 *                 output column per 128 consecutive input channels
 *                 (Section 2.2: weights are de-quantised on the fly to fp16
 *                 and multiplied with fp16 activations).
 *   LUT_COL8:     3-bit codes into one ascending 8-entry fp16 codebook per
 *                 output column: W_hat[k][n] = lut[n][c[k][n]] (the
 *                 clustering-based non-uniform quantisation of Section 5.2).
 */
typedef enum { DECDEC_W_UNIFORM_G128 = 0, DECDEC_W_LUT_COL8 = 1 } decdec_wfmt;

/* Residual formats in pinned CPU memory (Section 4.2).
 *   FP16:          R[K][N] fp16, each input-channel row contiguous.
 *   INT4_SYM_COL:  4-bit symmetric codes in [-7, 7], one fp16 scale per
 *                  output column: R_hat[k][n] = S[n] * q[k][n].  Row k is
 *                  N/2 contiguous bytes; byte j holds column 2j in its low
 *                  nibble and column 2j+1 in its high nibble, each a 4-bit
 *                  two's-complement integer.
 *   INT2_SYM_COL / INT8_SYM_COL: the same with 2-bit codes in [-1, 1] (four per
 *                  byte, column 4j+i in bits 2i..2i+1) or 8-bit codes in
 *                  [-127, 127] (one per byte): the variants of the paper's
 *                  residual bit-width study (Table 2).
 */
typedef enum {
    DECDEC_R_FP16 = 0,
    DECDEC_R_INT4_SYM_COL = 1,
    DECDEC_R_INT2_SYM_COL = 2,
    DECDEC_R_INT8_SYM_COL = 3
} decdec_rfmt;

typedef struct {
    int32_t K;      /* input channels  (d_in),  multiple of 128 */
    int32_t N;      /* output channels (d_out), multiple of 64  */
    int32_t wbits;  /* 3 or 4 (LUT_COL8: 3) */
    int32_t wfmt;   /* decdec_wfmt */
    int32_t rfmt;   /* decdec_rfmt */
} decdec_desc;

typedef struct decdec_ws decdec_ws; /* opaque workspace */

/* ------------------------------------------------------------------ set-up */

/* Allocates everything the hot path needs for problems up to (maxK, maxN)
 * with up to maxk salient channels: a side stream and two events for the
 * overlap of Section 4.1, the sc_indices / x[sc_indices] buffer of
 * maxk*(4+2) bytes (Section 4.3 "GPU Memory Overhead"), and one 64-bit
 * accumulator per output column (8 maxN bytes) into which the base GEMV and
 * the residual kernel add.  One workspace can be reused for every layer. */
int decdec_ws_create(int32_t maxK, int32_t maxN, int32_t maxk, decdec_ws** out);
int decdec_ws_destroy(decdec_ws* ws);
/* Size in bytes of the sc_indices + x[sc_indices] buffer for k channels: the
 * only extra GPU memory of the paper's kernel (Section 4.3: 1433 channels ->
 * 8.6 KB). */
size_t decdec_sc_buffer_bytes(int32_t k);
/* Size in bytes of the fp32 partial rows that a workspace for maxN output
 * columns allocates when decdec_ws_set_inkernel_accumulate(ws, 0) is first
 * called (up to 16 rows of maxN floats from each of the two producers, 128 maxN
 * bytes); a workspace that keeps the default never holds them. */
size_t decdec_partial_buffer_bytes(int32_t maxN);
/* Device pointers to the selection of the most recent decdec_gemv call on
 * this workspace (valid once that call's work has run). */
int decdec_ws_last_selection(const decdec_ws* ws, const int32_t** idx_dev, const void** xsel_f16_dev);
/* Diagnostic, synchronous: waits for the whole device (the selection may have
 * been written from any stream) and copies the first k entries of that
 * selection to host arrays (either may be NULL). */
int decdec_ws_read_selection(const decdec_ws* ws, int32_t k, int32_t* idx_host, void* xsel_f16_host);

/* Number of wavefronts that share the selected rows of one 512-column segment
 * in the residual kernel, 1 .. 128 (the counterpart of n_tb in Section 4.4:
 * how many requests are in flight on the host link, at the price of compute
 * units the base GEMV cannot use); they are grouped into workgroups of 8, each
 * of which adds its rows' sum once per column.  0 restores the built-in choice (about
 * 128 wavefronts in the whole kernel, which saturate the link; more than about
 * 500 lower its rate).  Affects later calls on this workspace. */
int decdec_ws_set_fetch_split(decdec_ws* ws, int32_t row_split);

/* How one compensated GEMV (k > 0) is laid out on the GPU.  Every mode adds the
 * same terms in fp32; SERIAL and TWO_STREAMS give identical bits, FUSED may split
 * K over workgroups of another size, so its part sums may round differently.
 *   FUSED (default): one kernel whose first workgroups do steps 1-3 (selection,
 *     zero-copy fetch, residual GEMV) and whose other workgroups do the base
 *     GEMV, on the caller's stream (fp16 and 4-bit residuals; the 2- and 8-bit
 *     formats run as SERIAL).
 *   SERIAL: residual kernel and base GEMV kernel one after the other on the
 *     caller's stream.
 *   TWO_STREAMS: the arrangement of Section 4.1: steps 1-3 on the workspace's
 *     side stream, the base GEMV on the caller's stream, joined by events.
 * In every mode the two terms are added as decdec_ws_set_inkernel_accumulate
 * says. */
typedef enum { DECDEC_MODE_FUSED = 0, DECDEC_MODE_SERIAL = 1, DECDEC_MODE_TWO_STREAMS = 2 } decdec_mode;
int decdec_ws_set_mode(decdec_ws* ws, int32_t mode);

/* Where step 1 runs when decdec_gemv / decdec_gemv_multi select for themselves.
 * on = 0 (default): inside the residual kernel, every workgroup selecting for
 * itself (K <= 32768 and k <= 4096; larger problems use the selection kernel).
 * on = 1: always as a kernel of its own before the residual kernel.  The
 * selection is the same either way. */
int decdec_ws_set_separate_select(decdec_ws* ws, int32_t on);

/* How the part sums of the base GEMV (one per K-slice) and of the residual
 * kernel (one per slice of the selected channels) are added (step 4 of Section
 * 4.1; the paper adds with atomics from its fused kernel).
 *   on = 1 (default): with atomics, as in the paper, but in fixed point, so
 *     that the result does not depend on the order of arrival: every producer
 *     converts its fp32 part sum of a column to a multiple of 2^-30 and adds it
 *     to the column's 64-bit accumulator with one atomic, which also counts the
 *     producers; the one that arrives last rounds the sum to fp16, writes y and
 *     clears the accumulator.  No further launch.
 *   on = 0: the producers write fp32 partial rows and a small kernel of its own
 *     on the caller's stream, after both, converts and adds them the same way
 *     (same bits).  The first such call allocates the partial rows
 *     (decdec_partial_buffer_bytes; DECDEC_ENOMEM if that fails).
 * Range: a part sum is clamped to +-2^21 before conversion, 32 times beyond
 * what fp16 can hold: a clamped term leaves y infinite, as it would be without
 * the clamp, unless clamped terms of both signs meet in one column.  Inputs
 * are assumed finite; a NaN part sum counts as -2^21. */
int decdec_ws_set_inkernel_accumulate(decdec_ws* ws, int32_t on);

/* Number of 128-channel groups each wavefront of the base GEMV walks through
 * (how finely K is split over the chip); 0 restores the built-in choice. */
int decdec_ws_set_gemv_split(decdec_ws* ws, int32_t groups_per_wave);
/* Wavefronts per workgroup (4, 8 or 16; 0 restores the built-in choice) of the
 * base GEMV when it runs as a kernel of its own.  A workgroup adds the sums of
 * its wavefronts; when waves x groups_per_wave covers all of K and there is no
 * residual term (k == 0) the kernel writes y itself and nothing else is
 * launched. */
int decdec_ws_set_gemv_waves(decdec_ws* ws, int32_t waves_per_workgroup);
/* Host-side query, nothing is enqueued: the grid the base GEMV kernel of an
 * uncompensated call (k == 0) over K input channels and N_total output columns
 * (all matrices of a decdec_gemv_multi call together) would be launched with
 * under this workspace's current settings: number of workgroups, threads per
 * workgroup, K-slices per 64-column tile.  Any output pointer may be NULL.
 * Benchmarks use it to tell whether a stored profile still describes the
 * kernels that run. */
int decdec_ws_gemv_launch_shape(const decdec_ws* ws, int32_t K, int32_t N_total, int32_t* workgroups,
                                int32_t* threads, int32_t* k_slices);

/* Kernel timing for benchmarks.  capacity > 0 allocates that many sets of HIP
 * events (set-up call: allocates, synchronises) and makes every later
 * decdec_gemv / _idx / _multi call on this workspace attach a (start, stop)
 * event pair to each kernel it launches, which receive that dispatch's own
 * begin and end timestamps (the duration a kernel trace reports);
 * capacity == 0 turns it off and frees the events.  Calls beyond `capacity`
 * since the last read are not timed.  Do not capture a graph while on. */
int decdec_ws_set_profiling(decdec_ws* ws, int32_t capacity);
/* Synchronous: waits for the device, then returns per kernel class the summed
 * kernel durations in milliseconds (ms[4]) and the number of timed launches
 * (calls[4]); class 0: base GEMV, 1: selection, 2: residual fetch + residual
 * GEMV, 3: accumulate.  Starts over afterwards.  Either pointer may be NULL. */
int decdec_ws_read_profile(decdec_ws* ws, double* ms, int32_t* calls);
/* The same read-out (synchronous, starts over afterwards), but listing the
 * duration in milliseconds of every timed launch of one kernel class in call
 * order: at most `capacity` values go to ms_per_launch, *count_out receives how
 * many.  Lets a benchmark attribute launches to the shapes it issued. */
int decdec_ws_read_profile_launches(decdec_ws* ws, int32_t kernel_class, float* ms_per_launch, int32_t capacity,
                                    int32_t* count_out);

/* A workspace verifies every residual pointer once (one query of its memory
 * type and of the extent of its allocation, the first time a hot-path call
 * sees it) and remembers about 3000 of them; later calls only look it up, so
 * a decode step of any depth costs no query and may be captured into a graph.
 * Call this before freeing residual memory whose address may be reused for
 * something else: p == NULL forgets every pointer. */
int decdec_ws_forget_pointer(decdec_ws* ws, const void* p);
/* Diagnostic: number of pointer queries this workspace has made so far. */
int64_t decdec_ws_pointer_queries(const decdec_ws* ws);

/* ------------------------------------------------- host helpers (offline) */

/* Bytes of the library-private packed form of the K x N code matrix. */
size_t decdec_packed_bytes(const decdec_desc* d);
/* codes_KN: host uint8 [K][N], one code per byte (values < 2^wbits).
 * out_packed: host buffer of decdec_packed_bytes(d); copy it to the GPU and
 * pass it as Wq.  The packed layout is private to the library. */
int decdec_pack_weights(const decdec_desc* d, const uint8_t* codes_KN, void* out_packed);
/* Inverse of decdec_pack_weights (host), for checking. */
int decdec_unpack_weights(const decdec_desc* d, const void* packed, uint8_t* codes_KN);
/* codes: host int8 [K][N] in [-7,7] -> out: host bytes [K][N/2] in the
 * INT4_SYM_COL row format above. */
int decdec_pack_residual_int4(int32_t K, int32_t N, const int8_t* codes_KN, uint8_t* out);
/* The same for bits in {2, 4, 8}: codes in [-(2^(bits-1) - 1), 2^(bits-1) - 1],
 * out: host bytes [K][N * bits / 8]; N a multiple of 128 / bits. */
int decdec_pack_residual_int(int32_t K, int32_t N, int32_t bits, const int8_t* codes_KN, uint8_t* out);

/* ------------------------------------------------------------ hot path */

/* Step 1 of Section 4.1 with the exact Top-K of Section 5.2: writes the k
 * indices i with the largest |x_i| in ascending index order (a tie at the cut
 * goes to the lower index; |x| is ordered by the fp16 bit pattern with the
 * sign cleared, so -0 == +0 and NaN patterns rank above infinity) and, if
 * xsel_f16_dev is not NULL, x at those indices.
 *   x_f16_dev: dev fp16 [K], 16-byte aligned, K a multiple of 8, 8 <= K <= 65536;
 *   0 <= k <= K.
 *   idx_out_dev: dev int32 [k];  xsel_f16_dev: dev fp16 [k] or NULL.
 * k == 0 enqueues nothing. */
int decdec_select_topk(const void* x_f16_dev, int32_t K, int32_t k,
                       int32_t* idx_out_dev, void* xsel_f16_dev, void* stream);

/* Step 1 as the paper's kernel does it (Section 4.3, fast approximate Top-K):
 * x is cut into chunks of 1024 channels and every chunk contributes k_chunk
 * channels.  Inside a chunk |x| is scattered into 32 buckets with boundaries
 *   b_i = b0 - i (b0 - b15) / 15  (0 <= i <= 15),  b_i = b15 (31 - i) / 16  (15 <= i <= 30),
 * bucket 0 = |x| >= b0, bucket 31 = |x| < b_30; channels are gathered from
 * bucket 0 upwards and the bucket that overflows gives its lowest indices (the
 * paper picks at random there).  b0 >= b15 >= 0 come from calibration: b15 the
 * largest k-th largest |x| over calibration vectors, b0 the largest |x| seen.
 * The bucket of a value is computed in fp32 as
 *   |x| >= b0: 0;  |x| >= b15: clamp(ceil((b0 - |x|) / ((b0 - b15) / 15)), 1, 15);
 *   else: 31 - clamp(floor(|x| / (b15 / 16)), 0, 15).
 *   x_f16_dev: dev fp16 [K], 16-byte aligned, K a multiple of 1024; 0 <= k_chunk <= 1024.
 *   idx_out_dev: dev int32 [k_chunk * K / 1024], chunk after chunk, ascending
 *   inside a chunk (hence ascending overall); xsel_f16_dev: fp16 of the same
 *   length or NULL.  Feed the result to decdec_gemv_idx.  k_chunk == 0 enqueues nothing. */
int decdec_select_bucket(const void* x_f16_dev, int32_t K, int32_t k_chunk, float b0, float b15,
                         int32_t* idx_out_dev, void* xsel_f16_dev, void* stream);

/* The whole path (Section 4.1 steps 1-4 beside the base GEMV):
 *   y = W_hat x + R_hat[sc,:]^T x[sc],  sc = top-k of |x|.
 *   x_f16_dev      dev fp16 [K]
 *   Wq_dev         dev, packed by decdec_pack_weights (or decdec_quantize_uniform)
 *   scales_f16_dev dev fp16 [K/128][N]           (UNIFORM; ignored for LUT)
 *   zeros_or_lut   dev fp16 [K/128][N] zero points (UNIFORM) or fp16 [N][8] (LUT)
 *   R_pinned       fp16 [K][N] or integer codes [K][N*bits/8] in pinned host memory, read in
 *                  place over the host link (the paper's placement, Section 4.3), or in
 *                  device memory (a GPU with room for the residuals: the same kernels
 *                  then read the selected rows from HBM); may be NULL if k == 0
 *   R_scales_f16_dev fp16 [N] (integer residual formats only, else NULL): device memory, or pinned
 *                  host memory as in the paper (Section 4.2: all scales are fetched with the rows),
 *                  at the price of 2 N more bytes over the host link per call
 *   k              salient channels, 0 <= k <= min(K, maxk of ws)
 *   y_f16_dev      dev fp16 [N] out
 * By default the base GEMV and steps 1-3 run side by side inside one kernel on
 * `stream` (see decdec_ws_set_mode) and add their part sums themselves
 * (fp32 accumulation inside a workgroup, the workgroups' sums added in fixed
 * point, one rounding to fp16: decdec_ws_set_inkernel_accumulate); the result
 * does not depend on the order in which workgroups finish.  k == 0 equals the
 * plain quantised GEMV.
 * The call only enqueues kernels (plus, in TWO_STREAMS mode, event records and
 * waits on the workspace's second stream), so it may be captured into a HIP
 * graph.  The first call that sees a given R_pinned queries the pointer's
 * memory type and the extent of its allocation (two host-side runtime
 * queries, no stream work, so this too is legal during capture); every later
 * call finds it in the workspace's table (decdec_ws_forget_pointer).  Calls
 * that share a workspace must be ordered on one stream: they share its
 * accumulators and selection buffer.
 * Errors: DECDEC_EINVAL for null / misaligned / out-of-range arguments and for
 * a residual allocation shorter than K rows, DECDEC_EUNSUPPORTED
 * for a format combination that is not built, DECDEC_ENOTPINNED if R_pinned
 * is neither pinned host memory nor device memory, DECDEC_EHIP for a failed launch
 * (decdec_last_hip_error); nothing is enqueued when validation fails. */
int decdec_gemv(const decdec_desc* d, const void* x_f16_dev, const void* Wq_dev,
                const void* scales_f16_dev, const void* zeros_or_lut_f16_dev,
                const void* R_pinned, const void* R_scales_f16_dev,
                int32_t k, void* y_f16_dev, decdec_ws* ws, void* stream);

/* Same with the selection supplied by the caller (layers that share one x,
 * such as q/k/v or gate/up, select once): idx_dev int32 [k] ascending,
 * xsel_f16_dev fp16 [k] = x[idx].  Indices must lie in [0, K). */
int decdec_gemv_idx(const decdec_desc* d, const void* x_f16_dev, const void* Wq_dev,
                    const void* scales_f16_dev, const void* zeros_or_lut_f16_dev,
                    const void* R_pinned, const void* R_scales_f16_dev,
                    int32_t k, const int32_t* idx_dev, const void* xsel_f16_dev,
                    void* y_f16_dev, decdec_ws* ws, void* stream);

/* One weight matrix with its residual and its output, for decdec_gemv_multi. */
typedef struct {
    const decdec_desc* desc;
    const void* Wq_dev;               /* as in decdec_gemv */
    const void* scales_f16_dev;
    const void* zeros_or_lut_f16_dev;
    const void* R_pinned;
    const void* R_scales_f16_dev;
    void* y_f16_dev;                  /* dev fp16 [desc->N] out */
} decdec_linear;

/* Up to 4 linear layers that consume the same x (q/k/v, gate/up: the paper's
 * fused layer types of Section 4.4) in one pass: one selection, one launch of
 * each kernel over the concatenated output columns.  All descriptors must
 * agree in K, wbits, wfmt and rfmt; the sum of their N must not exceed the
 * workspace's maxN.  Each y_m equals what decdec_gemv would produce for
 * matrix m alone. */
int decdec_gemv_multi(int32_t count, const decdec_linear* linears, const void* x_f16_dev, int32_t k,
                      decdec_ws* ws, void* stream);

/* decdec_gemv for callers that cannot allocate: code running under HIP graph
 * capture before any workspace exists, tight serving loops, harnesses that
 * forbid hipMalloc.  Same computation and same kernels as decdec_gemv in its
 * default mode, but no workspace: the selection buffer and the per-column
 * accumulators live in a fixed array in the library's device image (280 KB, held
 * by every GPU the library runs on until the process ends).  The call
 * allocates nothing, on the host or on the device.
 *   Limits: N <= DECDEC_STATIC_MAX_N, k <= DECDEC_STATIC_MAX_SELECTED;
 *   beyond them the call returns DECDEC_ETOOLARGE and enqueues nothing.
 *   Other arguments, results and errors as for decdec_gemv.
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams without ordering between them) race.  The first
 * call on a GPU looks the array's address up; make it outside graph capture. */
#define DECDEC_STATIC_MAX_N 32768
#define DECDEC_STATIC_MAX_SELECTED 4096
int decdec_gemv_static(const decdec_desc* d, const void* x_f16_dev, const void* Wq_dev,
                       const void* scales_f16_dev, const void* zeros_or_lut_f16_dev,
                       const void* R_pinned, const void* R_scales_f16_dev,
                       int32_t k, void* y_f16_dev, void* stream);

/* ------------------------------------------------ offline, on the device */

/* Uniform min/max group-128 quantiser on the GPU (offline preparation; the
 * paper takes this step from third-party work, Section 5.2):
 *   s = fp16((max - min) / (2^b - 1)) (1 if 0), z = clip(rint(-min / s), 0, 2^b-1),
 *   q = clip(rint(w / s) + z, 0, 2^b-1), every operation in IEEE fp32;
 *   R = fp16(w - s (q - z)).
 *   W_f32_dev dev fp32 [K][N] in;  Wq_out_dev packed codes out;
 *   scales/zeros dev fp16 [K/128][N] out;  R_f16_out dev or pinned fp16 [K][N]
 *   out, or NULL. */
int decdec_quantize_uniform(const decdec_desc* d, const void* W_f32_dev, void* Wq_out_dev,
                            void* scales_f16_out_dev, void* zeros_f16_out_dev,
                            void* R_f16_out, void* stream);

/* R = W - W_hat for weights that are already quantised and packed (Section 3.1;
 * any base quantiser, as the paper applies the method on top of third-party
 * ones, Section 5.2): one fp32 subtraction per element, W_hat = s (q - z)
 * (exact in fp32) or the codebook entry.
 *   W_f32_dev dev fp32 [K][N];  Wq_dev / scales / zeros_or_lut as for decdec_gemv
 *   (scales NULL for LUT_COL8);  R_f32_out_dev dev fp32 [K][N] out. */
int decdec_residual_f32(const decdec_desc* d, const void* W_f32_dev, const void* Wq_dev, const void* scales_f16_dev,
                        const void* zeros_or_lut_f16_dev, void* R_f32_out_dev, void* stream);

/* The residual quantiser (Section 4.2; bits = 4 is the paper's, 2 and 8 the
 * other integer widths of Table 2): per output column n
 *   q[k][n] = clip(rint(R[k][n] / S[n]), -qmax, qmax),  qmax = 2^(bits-1) - 1,
 * S[n] the value of fp16(alpha max_k|R[k][n]| / qmax), alpha = 0.30, 0.31, ...,
 * 1.00, with the least sum_k (R - S q)^2 (a tie keeps the larger alpha; a
 * column whose scale rounds to 0 gets S = 1).  Every step is one IEEE fp64
 * operation and a column's error is summed over k in ascending order.
 *   R_f32_dev dev fp32 [K][N] in;  codes_out dev or pinned bytes [K][N*bits/8],
 *   the layout of decdec_pack_residual_int;  scales_f16_out_dev dev fp16 [N];
 *   N a multiple of 128 / bits. */
int decdec_quantize_residual(int32_t K, int32_t N, int32_t bits, const void* R_f32_dev, void* codes_out,
                             void* scales_f16_out_dev, void* stream);

/* ------------------------------------------------------------ diagnostics */
const char* decdec_strerror(int status);
int decdec_last_hip_error(void); /* hipError_t of the last failing HIP call on this thread */
/* DECDEC_OK if p is GPU-visible host memory, DECDEC_ENOTPINNED otherwise. */
int decdec_check_pinned(const void* p);
/* DECDEC_OK if p may serve as a residual pointer: pinned host memory or device memory. */
int decdec_check_residual_pointer(const void* p);

#ifdef __cplusplus
}
#endif
#endif /* DECDEC_H */
