/*
 * nq_binlr.h -- C ABI of the MI355X (gfx950) library for the forward pass of a
 * NanoQuant low-rank binary factorized linear layer.
 *
 * Operation (quantization scheme, Section 3.1, Eq. 1; restated with diagonal
 * matrices in Appendix F.5, "NanoQuant (Ours)"):
 *
 *     W^ = Diag(s_out) . U . V^T . Diag(s_in),   U in {-1,+1}^{d_out x r},
 *                                                V in {-1,+1}^{d_in  x r},
 *     y[b, :] = W^ . x[b, :]  evaluated as  s_out (.) ( U . ( V^T . ( s_in (.) x[b, :] ) ) )
 *
 * i.e. the two scale vectors act only at the input and output boundary and the
 * two binary products run back to back (Section 3.3, Step 2, last sentence).
 * s_out is the paper's output-channel scale s1, s_in its input-channel scale
 * s2.  There is no bias.
 *
 * Canonical packed sign format (the interchange format of this ABI).  The
 * paper fixes the polarity (Fig. 2(c): -1 -> bit 0, +1 -> bit 1) but neither
 * word size nor bit order; this library uses: row-major over the factor's
 * rows (U: d_out rows, V: d_in rows), packed along the rank axis, rank index
 * k lives in 32-bit word k/32 of its row at bit position k%32 counted from
 * the least significant bit, words little-endian, each row padded to a whole
 * word with 0 bits.  The layout in device memory is private to the library.
 *
 * Conventions
 *  - every function returns an int status (NQ_OK = 0, errors negative), never
 *    throws, never aborts;  nq_last_error_string() describes the most recent
 *    failure on the calling thread;
 *  - "host" / "device" is stated for every pointer;  the caller owns every
 *    buffer it passes in, the library copies what it keeps;
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Functions taking a stream only enqueue work and do not synchronise,
 *    unless stated otherwise;
 *  - batched activations are row-major contiguous: x[batch][d_in],
 *    y[batch][d_out].
 *  - a token whose input holds a NaN or an infinity yields NaN in every output
 *    of that token (other tokens are unaffected).
 */
#ifndef NQ_BINLR_H
#define NQ_BINLR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define NQ_OK             0
#define NQ_E_INVALID_ARG (-1)  /* a value is not acceptable (NaN sign, int8 not +-1, bad dtype, batch < 1 ...) */
#define NQ_E_SHAPE       (-2)  /* a dimension is < 1 or beyond what the kernels support */
#define NQ_E_ALIGN       (-3)  /* a device pointer is not 16-byte aligned */
#define NQ_E_NULL        (-4)  /* a required pointer is NULL */
#define NQ_E_UNSUPPORTED (-5)  /* valid request that this build does not implement */
#define NQ_E_HIP         (-6)  /* a HIP runtime call failed (see nq_last_error_string) */
#define NQ_E_TIMEOUT     (-7)  /* a bounded wait inside a kernel ran into its limit (nq_exec_status) */

/* element types */
#define NQ_I8   0   /* int8, values must be exactly -1 or +1 (pack input only) */
#define NQ_F32  1
#define NQ_F16  2   /* IEEE binary16 */
#define NQ_BF16 3
#define NQ_F64  4   /* IEEE binary64: nq_lb_admm.h and nq_probe_mfma only */

/* nq_binlr_create flags */
#define NQ_FLAG_DEFAULT      0u
#define NQ_FLAG_DECODE_VALU  1u  /* every batch runs the plain fp32 vector-ALU kernels instead of the
                                    fixed-point matrix-core kernels (slow; a second implementation
                                    kept for cross-checks and as the paper-style "mask + FMA" GEMV) */
#define NQ_FLAG_NO_PREFILL   2u  /* never take the dense MFMA path: a batch above 8 is run as chunks of 8
                                    through the streaming kernels (their accuracy, their cost per chunk) */

typedef struct nq_binlr_s* nq_handle;   /* one factorized layer resident on one GPU */
typedef struct nq_plan_s*  nq_plan;     /* a fixed list of independent forwards */
typedef struct nq_exec_s*  nq_exec;     /* a fixed list of layers run in dependency order by one launch */

/* Largest d_in, d_out or r accepted (exactness of the 32-bit accumulators). */
#define NQ_MAX_DIM 65536
/* Largest batch served by the streaming (decode) kernels in one pass. */
#define NQ_DECODE_MAX_BATCH 8
/* Batches at or above this take the dense matrix-core (prefill) path: its cost is flat up to
 * 64 tokens (one token tile) and, measured, never above that of two streaming passes. */
#define NQ_PREFILL_MIN_BATCH 9

/* ---- packing (Algorithm 1, PackBinary; Fig. 2(c)) -- host only, no GPU needed ---- */

/* Number of uint32 words of a packed [rows, cols] sign matrix: rows * ceil(cols/32). */
size_t nq_packed_words(int64_t rows, int64_t cols);

/* signs: host, [rows, cols] row-major of `dtype` (NQ_I8, NQ_F32, NQ_F16, NQ_BF16).
 * out_words: host, nq_packed_words(rows, cols) words, fully overwritten.
 * bit = 1 iff value >= 0 (both zeros -> +1), bit = 0 iff value < 0.
 * NaN, or an int8 other than +-1 -> NQ_E_INVALID_ARG (out_words unspecified). */
int nq_pack_signs(const void* signs, int dtype, int64_t rows, int64_t cols, uint32_t* out_words);

/* Exact inverse on the first `cols` bits of every row. out_pm1: host int8 [rows, cols]. */
int nq_unpack_signs(const uint32_t* words, int64_t rows, int64_t cols, int8_t* out_pm1);

/* The same packing on the GPU (Algorithm 1, PackBinary, for factors that already live in device
 * memory, e.g. the latent matrices at the end of Phase 3).
 * d_signs: device, [rows, cols] row-major of `dtype`;  d_words: device, nq_packed_words(rows, cols)
 * words, fully overwritten with the canonical format (identical to nq_pack_signs' output).
 * d_invalid: device int32 or NULL; incremented once for every NaN (or int8 other than +-1) met,
 * which is packed as bit 0 -- the caller clears it before and reads it after.
 * Asynchronous on `stream`; allocates nothing.  rows < 2^31, cols <= 65535 * 256. */
int nq_pack_signs_device(const void* d_signs, int dtype, int64_t rows, int64_t cols,
                         uint32_t* d_words, int32_t* d_invalid, void* stream);

/* ---- layer objects ---- */

/* Build a layer on the current HIP device.
 * U_words: host, canonical [d_out, ceil(r/32)];  V_words: host, canonical [d_in, ceil(r/32)];
 * s_out_fp16: host, d_out IEEE binary16 values;  s_in_fp16: host, d_in values.
 * x_dtype: NQ_F32, NQ_F16 or NQ_BF16;  y_dtype: NQ_F32 (default of the build's parity bar),
 * NQ_F16 or NQ_BF16: the fp32 result rounded once more, to nearest even (a value beyond the
 * fp16 range becomes infinity, as in IEEE conversion; the paper does not state an output
 * type, its models run in bf16/fp16).
 * Copies everything, rearranges the bits on the GPU, and synchronises the device.
 * Any r, d_in, d_out in [1, NQ_MAX_DIM] is accepted (tails are padded inside).
 * Workspace for batch <= NQ_DECODE_MAX_BATCH is allocated here. */
int nq_binlr_create(nq_handle* out, int64_t d_out, int64_t d_in, int64_t r,
                    const uint32_t* U_words, const uint32_t* V_words,
                    const uint16_t* s_out_fp16, const uint16_t* s_in_fp16,
                    int x_dtype, int y_dtype, uint32_t flags);

/* nq_binlr_create with all four inputs in device memory of the current device (canonical words as
 * written by nq_pack_signs_device, fp16 scales); same checks, same result. */
int nq_binlr_create_from_device(nq_handle* out, int64_t d_out, int64_t d_in, int64_t r,
                                const uint32_t* d_U_words, const uint32_t* d_V_words,
                                const uint16_t* d_s_out_fp16, const uint16_t* d_s_in_fp16,
                                int x_dtype, int y_dtype, uint32_t flags);

/* Three-scale variant -- the format of the low-rank binary methods the paper compares with
 * (DBF, LittleBit; Appendix F.4):
 *     W^ = Diag(s_out) . U . Diag(s_mid) . V^T . Diag(s_in),
 *     y  = s_out (.) ( U ( s_mid (.) ( V^T ( s_in (.) x ) ) ) ),     s_mid: r rank-wise scales.
 * s_mid_fp16: host, r IEEE binary16 values (finite, any sign), copied; NULL removes the scale again
 * (back to the two-scale layer of Eq. 1).  Every path applies it: the streaming kernels while they
 * quantise t, the dense path when it stores T.  Synchronises the device.  Call it before plans are
 * built on the handle (a plan keeps the layer's descriptors; the cached plan of
 * nq_binlr_forward_many is dropped here).  nq_binlr_weight_bytes then counts the 2r bytes too. */
int nq_binlr_set_mid_scale(nq_handle h, const uint16_t* s_mid_fp16);

/* Grow the per-layer workspace so that forwards with ANY batch <= max_batch allocate nothing
 * (the dense path's need is not monotone in the batch; the largest need up to max_batch is taken).
 * May allocate and synchronise. */
int nq_binlr_reserve(nq_handle h, int max_batch);
/* What has been reserved: the largest batch that allocates nothing, and the bytes of the dense
 * path's workspace held by the layer.  Either pointer may be NULL. */
int nq_binlr_reserved(nq_handle h, int* max_batch, size_t* workspace_bytes);

/* y = s_out (.) (U (V^T (s_in (.) x))) for `batch` tokens (Eq. 1).
 * x: device, [batch, d_in] of x_dtype;  y: device, [batch, d_out] of y_dtype; both 16-byte
 * aligned, must not overlap.  Asynchronous on `stream`.  Allocates nothing when
 * batch <= the reserved batch (otherwise it reserves first, which synchronises).
 * Not re-entrant on one handle (the handle's workspace is shared); different
 * handles may run concurrently on different streams.
 * batch <= 8: streaming kernels (exact integer accumulation); >= 9: dense MFMA path
 * (fp16 operands, fp32 accumulation), unless the layer was created with NQ_FLAG_NO_PREFILL. */
int nq_binlr_forward(nq_handle h, const void* x, void* y, int batch, void* stream);

/* nq_binlr_forward for callers that cannot allocate device memory or rely on a workspace the
 * library allocated for them: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bit-identical results for batch <=
 * NQ_DECODE_MAX_BATCH (larger batches: NQ_E_UNSUPPORTED), but the kernels' scratch memory (the
 * fixed-point copies of x' and t, the token constants, the intermediate t) is a static array of
 * NQ_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends,
 * instead of the layer's own workspace.  A layer and batch that need more (about
 * batch * 3.2 * (d_in + r) bytes: any BASELINE shape at batch 8 fits) -> NQ_E_SHAPE.  The call
 * allocates and frees nothing and clears nothing (every byte read was written earlier in the
 * same call).  Every call on one GPU uses that GPU's one array: calls that overlap in time on one
 * GPU (two streams, two threads) race; calls on one stream follow one another safely.
 * nq_binlr_read_intermediate does not see this call's t. */
#define NQ_STATIC_SCRATCH_BYTES (2u << 20)
int nq_binlr_forward_static(nq_handle h, const void* x, void* y, int batch, void* stream);

/* The same product for ANY batch through the streaming kernels only, in passes of up to 8 tokens
 * (exact integer accumulation of 24-bit fixed-point activations: the accuracy of a batch <= 8
 * forward, at the cost of one pass over the bits per 8 tokens) -- the per-call way to ask for the
 * exact path above batch 8, where nq_binlr_forward takes the fp16-operand dense path.
 * Pointers, types and stream as in nq_binlr_forward; allocates nothing. */
int nq_binlr_forward_exact(nq_handle h, const void* x, void* y, int batch, void* stream);

/* ---- scale gradients with the packed signs frozen (Section 3.4; Algorithm 1, Phase 3) ----
 * For a loss L with upstream gradient g = dL/dy ([batch, d_out]):
 *     dL/ds_out = sum_b g_b (.) z_b,                 z = U (V^T (s_in (.) x))        (the forward without s_out)
 *     dL/ds_in  = sum_b x_b (.) w_b,                 w = V (U^T (s_out (.) g))
 * z comes from nq_binlr_forward_unscaled, w from nq_binlr_forward_transposed_unscaled on the SAME
 * layer object (the transposed products read the resident bits; no second copy of the weights);
 * nq_scale_grad does the products and the sum over the batch. */

/* z = U (V^T (s_in (.) x)) [(.) s_mid where set]: the forward without its output scale.  Pointers
 * and types as in nq_binlr_forward (z has y_dtype).  Any batch, run as passes of up to 8 tokens through the
 * streaming kernels (exact integer accumulation).  Asynchronous on `stream`. */
int nq_binlr_forward_unscaled(nq_handle h, const void* x, void* z, int batch, void* stream);

/* w = V (s_mid (.) (U^T (s_out (.) g))): the layer's transpose applied to g without the input scale
 * (s_mid only where nq_binlr_set_mid_scale has set one).
 * g: device, [batch, d_out] row-major of the layer's y_dtype;  w: device, [batch, d_in] floats.
 * Any batch (passes of up to 8 tokens).  Sign products are exact and added in binary64 on the vector
 * ALU, each result is rounded once to fp32 (u = U^T(..) between the two products likewise).  The first
 * call on a layer allocates its workspace (and synchronises the device then); afterwards the call is
 * asynchronous on `stream`.  g and w must be 16-byte aligned. */
int nq_binlr_forward_transposed_unscaled(nq_handle h, const void* g, float* w, int batch, void* stream);

/* The gradient of a loss with respect to the layer's input, dL/dx = W^T g = s_in (.) w with w as above
 * (the layer is linear in x; Section 3.4 back-propagates through the frozen packed layers).
 * Same pointers, types, workspace and stream behaviour as nq_binlr_forward_transposed_unscaled. */
int nq_binlr_backward_input(nq_handle h, const void* g, float* dx, int batch, void* stream);

/* out[j] = sum_{b < batch} a[b][j] * b[b][j], j < n.  a, b: device, [batch, n] row-major of a_dtype /
 * b_dtype (NQ_F32, NQ_F16, NQ_BF16); out: device float [n].  fp64 accumulation, one rounding.
 * Asynchronous on `stream`; allocates nothing. */
int nq_scale_grad(const void* a, int a_dtype, const void* b, int b_dtype, int batch, int64_t n, float* out,
                  void* stream);

/* n independent forwards (same batch <= NQ_DECODE_MAX_BATCH) in four launches in total:
 * the streaming kernels walk a work list that covers all n layers, so small
 * layers do not pay one launch each.  hs/xs/ys: host arrays of n entries; xs[i]/ys[i]
 * device pointers as in nq_binlr_forward.  A handle may appear only once; several layers may
 * read the same x (the q, k, v or the gate, up projections of a decoder block: the seven projections shown in
 * Appendix D.3's figure), each scaling and quantising it with its own s_in.  Calls follow one another on
 * the stream, so a later call may read what an earlier one wrote.
 * At batch 1 a list whose launches would be short (a decoder block's few layers) runs as two
 * launches, the stage kernels quantising their own input; results are bit-identical either way.
 * The list is compiled into an internal plan; the plans of the 32 most recently used argument lists
 * are kept (compiling allocates and synchronises; replays do not), so a model may call this once per
 * group of layers.  The cache is emptied when a handle is destroyed or its rank-wise scale changed. */
int nq_binlr_forward_many(const nq_handle* hs, const void* const* xs, void* const* ys,
                          int n, int batch, void* stream);

/* The same, with the plan made explicit. */
int nq_plan_create(nq_plan* out, const nq_handle* hs, const void* const* xs, void* const* ys,
                   int n, int batch);
int nq_plan_forward(nq_plan p, void* stream);
/* Runs the plan once with a pair of HIP events bound to each of its kernels (start and stop of the kernel itself,
 * hipExtLaunchKernelGGL: the dispatch gaps between launches are not part of any entry, so the entries add up to less
 * than the step), waits for it, and returns the duration of each kernel in milliseconds:
 * ms[0] input quantisation, ms[1] stage 1 (t = V^T x'), ms[2] quantisation of t,
 * ms[3] stage 2 (y = s_out (.) U t).  Synchronises `stream`.  Where a stage quantises its own
 * input (batch-1 lists) there is no quantisation launch: its entry is 0 and the stage entry
 * covers both. */
int nq_plan_forward_timed(nq_plan p, void* stream, float ms[4]);
/* Debug: which schedule each of the plan's two stage launches uses.  w[0] stage 1, w[1] stage 2:
 * 1 = one wave per item, 4 / 16 = that many waves share a row block, 8 = the waves of a workgroup share an op's
 * input through LDS (batch 4..8), 9 = the same with the whole input resident in LDS (reductions of at
 * most 16 steps), 32 = short batch-1 launch with reductions of 4097..16384 elements in which every
 * workgroup (16 waves per row block) quantises the input for itself,
 * 33 / 34 = batch-1 launch whose waves quantise their own share of the input (one / four waves per
 * row block; reductions of at most 1024 / 4096 elements). */
int nq_plan_schedules(nq_plan p, int w[2]);
int nq_plan_destroy(nq_plan p);

/* ---- layers in dependency order, one launch (batch 1) ----
 * A decoder block -- the seven projections of Appendix D.3's figure, called in the order of the decode
 * harness of Appendix D.1: q, k, v | o | gate, up | down -- or a whole stack of blocks, run by ONE
 * persistent kernel: one workgroup per CU walks its share of the 2 x levels phases (stage 1 and stage 2
 * of every level) and hands t and y from phase to phase through device memory, without a launch or
 * a grid-wide barrier in between.  Results are bit-identical to nq_binlr_forward called layer by layer.
 *
 * hs / xs / ys: host arrays of n entries, layers listed level by level; level_of[i] >= 0, non-decreasing.
 * xs[i] (device, d_in elements of the layer's x_dtype) is EITHER memory that no layer of the list writes
 * OR exactly ys[j] of a layer j of an earlier level (same pointer, d_in(i) = d_out(j), x_dtype(i) =
 * y_dtype(j)): then layer i waits for layer j's output.  No other ordering exists: layers that do not
 * depend on one another through such a buffer may run in any order or together, whatever their level.
 * ys[i] (device, d_out elements of y_dtype) must not overlap one another nor any input except as said.
 * 16-byte alignment as in nq_binlr_forward; d_in, r <= 32768; a handle may appear once.
 * nq_exec_create allocates (descriptors, task lists, the hand-over buffers) and synchronises;
 * nq_exec_forward only enqueues one launch on `stream` and allocates nothing; it may be captured in a HIP
 * graph and replayed.  Launches of one executor must follow one another on one stream.
 * Every wait inside the kernel is bounded (option "exec_spin_limit_us", default 2 s): should the
 * grid ever not be resident as a whole (another kernel holding CUs), waits give up, every workgroup
 * leaves, and nq_exec_status -- which synchronises `stream` -- returns NQ_E_TIMEOUT once; the outputs
 * of that launch are then incomplete. */
int nq_exec_create(nq_exec* out, const nq_handle* hs, const void* const* xs, void* const* ys,
                   const int* level_of, int n);
int nq_exec_forward(nq_exec e, void* stream);
int nq_exec_status(nq_exec e, void* stream);
/* Debug: workgroups of the launch, tasks in their lists, LDS bytes per workgroup.  Pointers may be NULL. */
int nq_exec_info(nq_exec e, int* n_workgroups, int* n_tasks, size_t* lds_bytes);
int nq_exec_destroy(nq_exec e);
/* Host only (no GPU needed): the task lists nq_exec_create would build for layers of these shapes on
 * n_workgroups workgroups.  tasks_out: host, capacity x 7 int32 -- workgroup, phase (2 level + stage),
 * layer, stage (0: t = V^T x', 1: y = U t), first row block, row blocks, waves per row block -- in
 * phase order; NULL to only count.  *n_tasks = number of tasks. */
int nq_exec_plan_tasks(const int64_t* d_out, const int64_t* d_in, const int64_t* r, const int* level_of, int n,
                       int n_workgroups, int32_t* tasks_out, int capacity, int* n_tasks);

int nq_binlr_destroy(nq_handle h);

/* Bytes of the stored factorization: r(d_in+d_out)/8 + 2(d_in+d_out), i.e. the bit count
 * r(n+m) + 16(n+m) of Appendix F.5 divided by 8 (padding not counted); with a rank-wise scale
 * 2r bytes more (r(n+m) + 16(n+r+m) bits, Appendix F.4). 0 for NULL. */
size_t nq_binlr_weight_bytes(nq_handle h);

/* Debug: number of device slabs (the large allocations layers are carved from) the library holds now. */
int nq_debug_slab_count(void);

/* Debug: convert the device-resident bits back to canonical words (host buffers sized as
 * in nq_binlr_create).  Synchronises.  Either pointer may be NULL to skip that factor. */
int nq_binlr_export_words(nq_handle h, uint32_t* U_words, uint32_t* V_words);

/* Debug: copy the intermediate t = V^T (s_in (.) x) of the most recent batch<=8 forward
 * on this handle to host float32 [batch, r].  Synchronises the device. */
int nq_binlr_read_intermediate(nq_handle h, float* t_host, int batch);

/* ---- measurement aids (not part of the forward path) ----
 * What this GPU attains on the two resources the roofline figures are priced against, so that a
 * benchmark can report its results against measured as well as nominal peaks. */

/* Streams a private buffer of `bytes` (>= 64 MiB; several times the 256 MB last-level cache for an
 * HBM figure) `iters` times through a read-only kernel and returns the rate in GB/s (1e9 bytes).
 * prewarm_ms (0..1000): about that many milliseconds of the same load run untimed first -- the chip
 * changes its power state a few milliseconds into a sustained load, and the rate with it.
 * Allocates and frees its buffer, runs on the default stream, synchronises. */
int nq_probe_hbm_read(size_t bytes, int iters, int prewarm_ms, double* gb_per_s);
/* A register-resident loop of dense matrix-core instructions on every CU: dtype NQ_F16 (fp16 operands,
 * fp32 accumulation; the prefill path's instruction) or NQ_I8 (int8, int32 accumulation; the decode
 * path's) or NQ_F64 (binary64, the LB-ADMM products').  Returns 1e12 operations per second (one
 * multiply-add = 2).  Synchronises. */
int nq_probe_mfma(int dtype, double* tera_ops_per_s);

/* ---- tuning options (process-wide) ----
 * Integers that steer the library's choice of schedules and tilings; every one has a measured
 * default and none changes a result beyond the documented tolerances -- with ONE exception:
 * "two_slice_b8" (off by default) makes plans created at batch 6..8 feed their shared-input
 * launches 16-bit instead of 24-bit fixed point (faster; about 3e-4 of the largest output instead
 * of 2e-6, and about 2e-3 -- outside this build's 1e-3 bar -- for inputs with outlier channels
 * 20 times the rest).  Names: "slab_mb",
 * "force_w", "split_steps", "selfq4_min_steps", "share_steps", "share_min_batch", "stream_steps",
 * "schedule_full", "fuse_max_mb", "no_fuse", "no_selfq", "no_selfq_c2", "no_resident",
 * "no_quant_wave", "pf_splits1", "pf_splits2", "pf_tg1", "pf_tg2", "pf_ks1", "pf_ks2", "pf_verbose",
 * "exec_spin_limit_us", "no_small_layer", "small_layer_kb", "dgemm_tile", "admm_no_overlap",
 * "two_slice_b8", "admm_no_prio", "admm_product_mode", "admm_inline_svid",
 * "admm_no_fused_step" (see the source for the meaning of each).  value < 0 restores the default.
 * The environment variable NQ_<NAME IN CAPITALS> gives an option its initial value; it is read once,
 * when the library first consults an option, never on a launch path.  Plans keep the schedules
 * chosen when they were created.  Not thread-safe against forwards running at the same time.
 * Unknown name -> NQ_E_INVALID_ARG. */
int nq_set_option(const char* name, int value);
/* *value = the option's current value, -1 when it is unset (built-in default applies). */
int nq_get_option(const char* name, int* value);

const char* nq_status_string(int status);
const char* nq_last_error_string(void);

#ifdef __cplusplus
}
#endif
#endif /* NQ_BINLR_H */
