// Internal declarations shared by the translation units of libnq_binlr (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <string>
#include "nq_binlr.h"

namespace nq {

// ---- device bit layout ("sign tiles") ------------------------------------------------------
// A sign matrix A[M][N] (M output rows, N = reduction length; A = V^T for stage 1, A = U for
// stage 2 of the two-stage product of Section 3.3 / Appendix E.2) is cut into tiles of
// 128 rows x 64 reduction columns = 1 KiB.  Tile (rb, st) starts at word (rb*n_steps + st)*256.
// Inside a tile, lane l of a wavefront owns words 4l..4l+3 (one 16-byte load).  In word v of
// lane l, bit 8*b + p  (byte b = 0..3, bit-in-byte p = 0..7) is the sign bit of
//     A[rb*128 + 16*p + (l & 15)][st*64 + 16*(l >> 4) + 4*v + b]      (1 -> +1, 0 -> -1).
// Masking a word with 0x01010101 << p therefore yields four int8 values in {0, 2^p} that are
// exactly the A operand (row l&15, depth 16*(l>>4) + 4v + b) of one 16x16x64 int8 MFMA for the
// 16 rows of bit plane p.  Rows >= M and columns >= N hold 0 bits.
constexpr int kTileRows = 128;
constexpr int kTileCols = 64;
constexpr int kTileWords = 256;

// ---- fixed-point activations ---------------------------------------------------------------
// The streaming kernels contract exact integers.  Each token's vector v (x' = s_in (.) x for
// stage 1, t for stage 2) is written as v_j ~= step * q_j with step a power of two chosen from
// the token's max |v_j| so that |q_j| <= 2^22, and q_j is split into three signed bytes
// q = 65536*hi + 256*mid + lo.  A token occupies three MFMA columns (hi, mid, lo) of a group of 16:
// five tokens per group; tokens 0..4 are columns 0..14 of group 0, tokens 5..7 columns 0..8 of group 1.
constexpr int kSlices = 3;
// Position, in 16-byte pieces inside a token's quantised vector, of slice `slice` of chunk `chunk` (16
// reduction indices): a 64-column step = 4 chunks = 12 pieces, ordered slice-major inside the step.
__host__ __device__ inline int bq_piece(int chunk, int slice) { return (chunk >> 2) * 12 + slice * 4 + (chunk & 3); }

// Per token, written by the quantisation: with step the token's power-of-two quantisation step and
// sum_q = sum_j q_j, a stage output is  (2 sum_n b_n q_n - sum_q) step = fma(sum_n b_n q_n, two_step, neg_qs).
// Both constants are exact (scalings of an exact integer by a power of two); two_step is NaN when
// the token holds a non-finite value, which makes every output of the token NaN.
struct QMeta {
    double two_step;  // 2 step
    double neg_qs;    // -sum_q step
};

struct QuantDesc {
    const void* x;           // device [batch][x_stride]
    const uint16_t* scale;   // device fp16 [N] or nullptr (no scaling)
    uint8_t* bq;             // device [batch][n_steps][3 slices][4 chunks][16] signed bytes (bq_piece)
    QMeta* meta;             // device [batch]
    int N;                   // real length
    int n_chunks;            // 16-element chunks including padding (= 4 * n_steps)
    int x_stride;            // elements between tokens
    int dtype;               // NQ_F32 / NQ_F16 / NQ_BF16
    int mag_exp;             // |q| <= 2^mag_exp: 22 (three byte slices; also when 0) or 14 (the top slice stays zero)
};

struct StageDesc {
    const uint32_t* tiles;       // sign tiles of A
    const uint8_t* bq;           // quantised input of this stage
    const QMeta* meta;
    const uint16_t* out_scale;   // fp16 [M] or nullptr
    void* out;                   // [batch][out_stride] elements of out_dtype
    int M;                       // real rows
    int n_steps;                 // 64-column steps
    int out_stride;
    int out_dtype;               // NQ_F32 (t, and y by default), NQ_F16 or NQ_BF16 (y)
};

// One unit of streaming work: a run of 128-row blocks of one op, each over its whole reduction length.
// Everything the wave needs before its first tile load sits in the item itself (one fetch).
struct WorkItem {
    const uint32_t* tiles;   // first tile of this row block
    const uint8_t* bq;       // quantised input of the op
    int n_steps;
    int op;                  // index into the StageDesc array (epilogue fields)
    int rb;                  // first row block of the item
    int n_rb;                // consecutive row blocks in the item (1 for the split schedule)
};

// One workgroup of the fused schedule: a row block of an op, with the op's descriptors copied in,
// so that the workgroup starts after a single fetch.
struct FusedItem {
    QuantDesc q;
    StageDesc s;
    int rb;
    int pad[3];
};

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }
inline int64_t n_rowblocks(int64_t M) { return (M + kTileRows - 1) / kTileRows; }
// the reduction is padded to a multiple of 4 steps (256 columns) so that the prefetch ring of the
// stream kernel stays in phase across row blocks; padding tiles hold 0 bits and quantised zeros
inline int64_t n_steps(int64_t N) { return (N + 4 * kTileCols - 1) / (4 * kTileCols) * 4; }
inline size_t tile_words(int64_t M, int64_t N) { return (size_t)n_rowblocks(M) * n_steps(N) * kTileWords; }

// ---- tuning options ------------------------------------------------------------------------
// Process-wide integers that steer the choice of schedules and tilings (the tests use them to run
// schedules built for large launches on small inputs; the defaults are the measured choices).
// An option is "unset" (-1: the built-in default applies) until nq_set_option gives it a value;
// the NQ_<NAME> environment variables are read ONCE, when the library first looks at an option, and
// never on a launch path.
enum Opt {
    OPT_SLAB_MB,            // size of the device slabs layers are carved from (default 512)
    OPT_FORCE_W,            // 1 / 4 / 16: schedule of the stage launches
    OPT_SPLIT_STEPS,        // reduction length from which a launch is split four ways (33 at batch 1, 64 above)
    OPT_SELFQ4_MIN_STEPS,   // shortest reduction of a launch whose four-wave row blocks quantise their own input (48)
    OPT_SHARE_STEPS,        // reduction length from which the shared-input kernel is taken (32)
    OPT_SHARE_MIN_BATCH,    // smallest batch that takes it (4)
    OPT_STREAM_STEPS,       // steps a stream item chains (16; 64 with two column groups)
    OPT_SCHEDULE_FULL,      // row blocks from which a launch counts as filling the chip (8 per CU)
    OPT_FUSE_MAX_MB,        // tile megabytes up to which a batch-1 plan launch takes the 16-wave fused kernel (24; 0: never)
    OPT_NO_FUSE,            // flag: no launch takes the 16-wave fused kernel
    OPT_NO_SELFQ,           // flag: no launch takes the one- and four-wave self-quantising kernels
    OPT_NO_SELFQ_C2,        // flag: one wave per row block quantises its own input only up to 16 steps
    OPT_NO_RESIDENT,        // flag: batch 6..8 never takes the resident-input variant of the shared kernel
    OPT_NO_QUANT_WAVE,      // flag: short vectors are quantised by the workgroup kernel too
    OPT_PF_SPLITS1, OPT_PF_SPLITS2,     // split count of the two prefill GEMMs
    OPT_PF_TG1, OPT_PF_TG2,             // token groups per workgroup tile (2 or 4)
    OPT_PF_KS1, OPT_PF_KS2,             // halves of the reduction taken inside a workgroup (1 or 2)
    OPT_PF_VERBOSE,         // flag: print the chosen prefill tiling
    OPT_EXEC_SPIN_LIMIT_US, // wall-clock limit, in microseconds, of every wait inside the dependent-layer executor (2 s)
    OPT_NO_SMALL_LAYER,     // flag: a lone small layer at batch 1 never takes the one-workgroup, one-launch kernel
    OPT_SMALL_LAYER_KB,     // packed size (KiB, both factors) up to which it does (160)
    OPT_DGEMM_TILE,         // tile of the binary64 product: 1 = 128 x 128, 2 = 128 x 64, 3 = 64 x 64 (default: by size)
    OPT_ADMM_NO_OVERLAP,    // flag: LB-ADMM runs the product with W on the caller's stream instead of beside the factorisation
    OPT_TWO_SLICE_B8,       // flag: plans at batch 6..8 run their shared-input launches on 16-bit fixed point (two byte slices)
    OPT_ADMM_NO_PRIO,       // flag: the kernels of LB-ADMM's factorisation chain keep the default wave priority
    OPT_ADMM_PRODUCT_MODE,  // 1: LB-ADMM's product with W keeps two workgroups per CU also beside the factorisation (default 0: one)
    OPT_ADMM_INLINE_SVID,   // flag: LB-ADMM runs the SVID of a factor on the caller's stream, before the next factor's update starts
    OPT_ADMM_NO_FUSED_STEP, // flag: LB-ADMM's factorisation launches the trailing update and the next diagonal block one after the other
    OPT_COUNT
};
int opt(Opt o);                                        // -1 when unset
inline int opt_or(Opt o, int dflt) { const int v = opt(o); return v >= 0 ? v : dflt; }
inline bool opt_flag(Opt o) { return opt(o) > 0; }

// A launch of the streaming path that is being timed carries a pair of events bound to the kernel itself
// (hipExtLaunchKernelGGL): their difference is the kernel's own execution time, what a profiler reports for it.
// Events recorded between launches would include the dispatch gaps and the event markers (two such events with
// nothing between them are 5 us apart).  nq_plan_forward_timed sets the pair for one launch at a time, on its thread.
struct LaunchTiming {
    hipEvent_t start = nullptr, stop = nullptr;
};
extern thread_local LaunchTiming g_launch_timing;
#define NQ_LAUNCH(kernel, grid, block, lds, s, ...)                                                              \
    do {                                                                                                         \
        if (nq::g_launch_timing.start)                                                                           \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, s, nq::g_launch_timing.start, nq::g_launch_timing.stop, 0, \
                                  __VA_ARGS__);                                                                  \
        else                                                                                                     \
            hipLaunchKernelGGL(kernel, grid, block, lds, s, __VA_ARGS__);                                        \
    } while (0)

// ---- error plumbing ------------------------------------------------------------------------
void set_error(const std::string& msg);
int hip_fail(hipError_t e, const char* what, const char* file, int line);
#define NQ_HIP(call)                                                        \
    do {                                                                    \
        hipError_t e__ = (call);                                            \
        if (e__ != hipSuccess) return ::nq::hip_fail(e__, #call, __FILE__, __LINE__); \
    } while (0)

// ---- output conversion (device code) ---------------------------------------------------------
#if defined(__HIPCC__)
// fp32 -> bf16 bits, round to nearest even; NaN stays NaN (quiet): the hardware's conversion (v_cvt_pk_bf16_f32),
// one instruction where the integer arithmetic for it takes six
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
// fp32 -> fp16 bits, round to nearest even (overflow gives infinity, as IEEE conversion does)
__device__ __forceinline__ uint16_t float_to_f16_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }
__device__ __forceinline__ uint16_t float_to_out16(float f, int dtype)
{
    return dtype == NQ_BF16 ? float_to_bf16_bits(f) : float_to_f16_bits(f);
}
// element `idx` of an output array of type `dtype` in global memory
// `streamed`: a final output, written once and not read back by the next launch -- stored
// non-temporal, so that it leaves the cache while the kernel still streams instead of waiting, dirty,
// for the write-back at the kernel's end (stage 2 of the 1024-layer pool: 100 -> 97.5 us).  The
// intermediate t, which the next launch reads, stays a plain store.
__device__ __forceinline__ void store_out(void* base, int dtype, size_t idx, float v, bool streamed = false)
{
    typedef __attribute__((address_space(1))) float* gptr_of32;
    typedef __attribute__((address_space(1))) uint16_t* gptr_ou16;
    if (streamed) {
        if (dtype == NQ_F32) __builtin_nontemporal_store(v, (gptr_of32)base + idx);
        else __builtin_nontemporal_store(float_to_out16(v, dtype), (gptr_ou16)base + idx);
    } else {
        if (dtype == NQ_F32) ((gptr_of32)base)[idx] = v;
        else ((gptr_ou16)base)[idx] = float_to_out16(v, dtype);
    }
}
#endif

// What the streaming kernels of one layer need beyond its inputs and outputs: the fixed-point copies
// of x' and t, their per-token constants, and the intermediate t.
struct DecodeWorkspace {
    uint8_t* bq_x;
    uint8_t* bq_t;
    QMeta* meta_x;
    QMeta* meta_t;
    float* t;             // [batch][t_stride]
    int t_stride;
};

}  // namespace nq

// ---- a layer resident on one GPU (the object behind nq_handle) ------------------------------
struct Slab;
struct nq_binlr_s {
    int64_t d_out, d_in, r;
    int x_dtype, y_dtype;
    uint32_t flags;
    int device;
    // weights (one allocation)
    void* w_alloc;
    size_t w_bytes;
    Slab* w_slab;
    uint32_t* vt_tiles;   // A = V^T : M = r,     N = d_in
    uint32_t* u_tiles;    // A = U   : M = d_out, N = r
    uint16_t* s_in;
    uint16_t* s_out;
    uint16_t* s_mid;      // rank-wise scale of the three-scale variant, fp16 [r padded to 128], or nullptr
    int mid_exp;          // ceil(log2(max |s_mid|)): keeps the dense path's fp16 intermediate in range
    // decode workspace (one allocation, sized for NQ_DECODE_MAX_BATCH, never reallocated)
    void* ws_alloc;
    size_t ws_bytes;
    Slab* ws_slab;
    nq::DecodeWorkspace ws;
    // prefill workspace (grown by reserve)
    void* pf_alloc;
    size_t pf_bytes;
    int pf_batch;
    // workspace of the transposed products (allocated by their first call)
    void* tp_alloc;
    size_t tp_bytes;
};


namespace nq {

// ---- launchers (nq_decode.hip) -------------------------------------------------------------
int launch_repack(const uint32_t* d_canon, int64_t wpr, bool transposed, int64_t M, int64_t N,
                  uint32_t* d_tiles, hipStream_t s);
int launch_export(const uint32_t* d_tiles, int64_t wpr, bool transposed, int64_t M, int64_t N,
                  uint32_t* d_canon, hipStream_t s);
int launch_pack_signs(const void* d_signs, int dtype, int64_t rows, int64_t cols, uint32_t* d_words, int* d_invalid,
                      hipStream_t s);
// single op (descriptor by value) or many (device arrays)
int launch_quantize(const QuantDesc* d_descs, const QuantDesc& single, int n_ops, int max_chunks, int batch,
                    hipStream_t s);
int stage_schedule(int n_rb_total, int mean_steps, int batch);
int stream_target_steps(int batch);
int stream_max_rbs(int batch);           // row blocks one stream item may chain (bounded by its LDS output buffer)
#ifndef NQ_SHARE_WAVES
#define NQ_SHARE_WAVES 4
#endif
constexpr int kShareWaves = NQ_SHARE_WAVES;    // waves of a workgroup of the shared-input kernel
// LDS one such workgroup may take: with four waves two workgroups share a CU (one streams while
// the other stages its input or flushes its results), with eight a workgroup has the CU to itself
constexpr int kShareLdsBytes = (kShareWaves <= 4 ? 80 : 160) * 1024 - 1024;
constexpr int kSharedSchedule = 8;       // stage_schedule()'s value for the workgroup-shared-input kernel
constexpr int kSharedResidentSchedule = 9;   // the same kernel with the whole input resident in LDS (reductions <= 16 steps)
// the two with 16-bit fixed point at batch 6..8: a token takes two MFMA columns, eight tokens one group of 16
constexpr int kSharedSchedule2 = 10, kSharedResidentSchedule2 = 11;
inline bool is_shared_schedule(int w) { return w >= kSharedSchedule && w <= kSharedResidentSchedule2; }
int shared_per_wave(int nst, int batch); // row blocks per wave of an item of that kernel
// w = 1: stream kernel (items are runs of rbs_per_item row blocks); w = 4 / 16: split kernel (one row block
// per item); w = kSharedSchedule: shared-input kernel (items of up to kShareWaves x shared_per_wave row blocks)
int launch_stage(const StageDesc* d_descs, const StageDesc& single, const WorkItem* d_items, int n_items,
                 int w, int rbs_per_item, int batch, hipStream_t s);
bool fused_fits(int nst, int batch);     // the quantised input of a stage fits the LDS of the fused kernel
int launch_fused(const QuantDesc& q, const StageDesc& sd, hipStream_t s);
constexpr int kFusedSchedule = 32;       // plan schedule code: a stage and its quantisation in one launch (batch 1)
int launch_fused_list(const FusedItem* d_items, int n_items, int max_steps, hipStream_t s);
// plan schedule codes: batch-1 launches with the quantisation done by the waves of the stage kernel
// themselves (stage_selfq_kernel<1> / <4>: one or four waves per row block)
constexpr int kSelfqSchedule1 = 33, kSelfqSchedule4 = 34;
bool selfq_fits(int w, int max_steps, int min_steps, int batch);
int selfq_width(int max_steps, int min_steps, int batch);    // for launches that do not fill the chip; 0: none
int launch_selfq(const FusedItem* d_items, int n_items, const QuantDesc& q1, const StageDesc& s1, int w, int max_steps,
                 hipStream_t s);
int launch_scale_grad(const void* a, int a_dtype, const void* b, int b_dtype, int batch, int64_t n, float* out,
                      hipStream_t s);
int launch_valu_gemv(const uint32_t* tiles, const void* x, int x_dtype, int x_stride, const uint16_t* in_scale,
                     const uint16_t* out_scale, void* out, int out_dtype, int out_stride, int64_t M, int64_t N,
                     int batch, hipStream_t s);
int device_cu_count();
int schedule_full_rowblocks();
int shared_min_batch();          // smallest batch that takes the shared-input kernel in launches that fill the chip            // row blocks from which a launch counts as filling the chip

// ---- launchers (nq_transposed.hip) -----------------------------------------------------------
size_t gemv_t_partial_bytes(int64_t M, int64_t N, int batch);
int launch_gemv_t(const uint32_t* tiles, int64_t M, int64_t N, const void* in, int in_dtype, int in_stride, const uint16_t* in_scale,
                  const uint16_t* out_scale, void* out, int out_dtype, int out_stride, int batch, double* partial, hipStream_t s);

// ---- launchers (nq_exec.hip) ---------------------------------------------------------------
bool small_layer_fits(nq_handle h, int batch);
int launch_small_layer(nq_handle h, const DecodeWorkspace& w, const void* x, void* y, bool unscaled, hipStream_t s);

// ---- launchers (nq_prefill.hip) ------------------------------------------------------------
struct PrefillArgs {
    const uint32_t* vt_tiles;   // stage-1 sign tiles (A = V^T)
    const uint32_t* u_tiles;    // stage-2 sign tiles (A = U)
    const uint16_t* s_in;
    const uint16_t* s_out;
    const uint16_t* s_mid;      // rank-wise scale (fp16, padded to whole row blocks with zeros) or nullptr
    int mid_exp;                // |s_mid| <= 2^mid_exp
    const void* x;
    void* y;
    void* workspace;            // device, prefill_workspace_bytes()
    int64_t d_out, d_in, r;
    int batch;
    int x_dtype, y_dtype;
};
size_t prefill_workspace_bytes(int64_t d_out, int64_t d_in, int64_t r, int batch);
int launch_prefill(const PrefillArgs& a, hipStream_t s);

}  // namespace nq
