// Streaming (decode, batch <= 8) kernels of the two-stage binary product
//     t = V^T (s_in (.) x),   y = s_out (.) (U t)          (Section 3.1 Eq. 1; Appendix E.2, GEMV)
// for gfx950.  Both stages are the same operation out[m] = sum_n A[m][n] v[n] with A a sign
// matrix stored as 1 bit per entry, so one kernel serves both.
//
// Why the matrix cores in a GEMV: at 8 TB/s the chip receives 64e12 sign bits per second but
// issues only ~39e12 vector lane-operations per second, so any per-bit mask/select/add scheme
// is ALU-bound far below the memory roofline.  Here a loaded 32-bit word is turned into four
// int8 operands of a 16x16x64 int8 MFMA by ONE v_and_b32 (see the tile layout in nq_internal.h):
// 0.25 vector op per weight, and the additions happen in the matrix pipe.  Signs enter as
// b in {0,1}; sum_n (2b-1) v = 2 sum_n b v - sum_n v, with sum_n v precomputed per token.
// Activations are exact integers (3 signed bytes per value, power-of-two step), so the
// accumulation is exact and the only rounding is the fixed-point step itself.
#include <algorithm>

#include "nq_internal.h"
#include "nq_device.h"

namespace nq {

// ---------------------------------------------------------------------------------------------
// canonical words <-> sign tiles
// ---------------------------------------------------------------------------------------------
__global__ void repack_kernel(const uint32_t* __restrict__ canon, int64_t wpr, int transposed, int64_t M, int64_t N,
                              int64_t nsteps, uint32_t* __restrict__ tiles, size_t n_words)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_words) return;
    size_t tile = idx / kTileWords;
    int wi = (int)(idx % kTileWords);
    int lane = wi >> 2, v = wi & 3;
    int64_t rb = tile / nsteps, st = tile % nsteps;
    int g = lane >> 4, i16 = lane & 15;
    uint32_t word = 0;
    for (int b = 0; b < 4; ++b) {
        int64_t col = st * kTileCols + 16 * g + 4 * v + b;
        if (col >= N) continue;
        for (int p = 0; p < 8; ++p) {
            int64_t row = rb * kTileRows + 16 * p + i16;
            if (row >= M) continue;
            uint32_t bit = transposed ? (canon[col * wpr + (row >> 5)] >> (row & 31)) & 1u
                                      : (canon[row * wpr + (col >> 5)] >> (col & 31)) & 1u;
            word |= bit << (8 * b + p);
        }
    }
    tiles[idx] = word;
}

// one thread per canonical word
__global__ void export_kernel(const uint32_t* __restrict__ tiles, int64_t wpr, int transposed, int64_t M, int64_t N,
                              int64_t nsteps, uint32_t* __restrict__ canon, size_t n_canon_words)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n_canon_words) return;
    int64_t crow = idx / wpr, cw = idx % wpr;
    uint32_t word = 0;
    for (int bit = 0; bit < 32; ++bit) {
        int64_t ck = cw * 32 + bit;          // index along the canonical packed axis (rank)
        int64_t row = transposed ? ck : crow;
        int64_t col = transposed ? crow : ck;
        if (row >= M || col >= N) continue;
        int64_t rb = row / kTileRows, rr = row % kTileRows, st = col / kTileCols, cc = col % kTileCols;
        int p = (int)(rr >> 4), i16 = (int)(rr & 15), g = (int)(cc >> 4), v = (int)((cc & 15) >> 2), b = (int)(cc & 3);
        uint32_t w = tiles[((size_t)rb * nsteps + st) * kTileWords + (size_t)(g * 16 + i16) * 4 + v];
        word |= ((w >> (8 * b + p)) & 1u) << bit;
    }
    canon[idx] = word;
}

int launch_repack(const uint32_t* d_canon, int64_t wpr, bool transposed, int64_t M, int64_t N, uint32_t* d_tiles,
                  hipStream_t s)
{
    size_t nw = tile_words(M, N);
    unsigned blocks = (unsigned)((nw + 255) / 256);
    hipLaunchKernelGGL(repack_kernel, dim3(blocks), dim3(256), 0, s, d_canon, wpr, transposed ? 1 : 0, M, N,
                       n_steps(N), d_tiles, nw);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

int launch_export(const uint32_t* d_tiles, int64_t wpr, bool transposed, int64_t M, int64_t N, uint32_t* d_canon,
                  hipStream_t s)
{
    // canonical matrix has (transposed ? N : M) rows of wpr words
    size_t nw = (size_t)(transposed ? N : M) * wpr;
    unsigned blocks = (unsigned)((nw + 255) / 256);
    hipLaunchKernelGGL(export_kernel, dim3(blocks), dim3(256), 0, s, d_tiles, wpr, transposed ? 1 : 0, M, N,
                       n_steps(N), d_canon, nw);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// ---------------------------------------------------------------------------------------------
// fixed-point quantisation of one token's vector (step a1 of the path when `scale` is given)
// grid = (n_ops, batch), block = NT (256 / 512 / 1024 for vectors up to 8192 / 16384 / longer: a workgroup
// is one token, and short vectors are latency-bound).  A thread owns 16-element chunks (one 16-byte
// group of the MFMA B operand per slice); up to kQuantHeld chunks stay in registers between the
// max pass and the rounding pass, longer vectors are read twice.
// ---------------------------------------------------------------------------------------------
constexpr int kQuantHeld = 2;

// STREAMED: the quantised bytes are written around the cache (non-temporal).  Measured on the pool of
// 1024 4096x4096 r=1024 layers: step 226 -> 213 us at batch 2, 261 -> 257 us at batch 4, but 382 -> 387 us at
// batch 8; taken for batch <= 5.
template <int kQuantThreads, bool STREAMED>
__global__ void __launch_bounds__(kQuantThreads)
quantize_kernel(const QuantDesc* __restrict__ descs, QuantDesc single, int batch)
{
    __shared__ float smf[kQuantThreads / 64];
    __shared__ double smd[kQuantThreads / 64];
    __shared__ int sm_bad;
    const QuantDesc d = descs ? descs[blockIdx.x] : single;
    const int tok = blockIdx.y;
    const int64_t base = (int64_t)tok * d.x_stride;
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    // 16-byte vector loads need every token row (and the row start) to be 16-byte aligned
    const int esz = d.dtype == NQ_F32 ? 4 : 2;
    const bool vec = (((size_t)d.x_stride * esz) & 15) == 0;
    const bool held = d.n_chunks <= kQuantThreads * kQuantHeld;
    if (tid == 0) sm_bad = 0;
    __syncthreads();

    // pass 1: max |v|; NaN/Inf is remembered separately (fmaxf drops NaN)
    float hv[kQuantHeld][16];
    float m = 0.f;
    int bad = 0;
    if (held) {
#pragma unroll
        for (int k = 0; k < kQuantHeld; ++k) {
            const int c = tid + k * kQuantThreads;
            if (c < d.n_chunks) {
                load_chunk16(d, base, c, vec, hv[k]);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float a = fabsf(hv[k][i]);
                    if (!(a <= 3.0e38f)) bad = 1;
                    m = fmaxf(m, a);
                }
            }
        }
    } else {
        for (int c = tid; c < d.n_chunks; c += kQuantThreads) {
            float v[16];
            load_chunk16(d, base, c, vec, v);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float a = fabsf(v[i]);
                if (!(a <= 3.0e38f)) bad = 1;
                m = fmaxf(m, a);
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((tid & 63) == 0) smf[wave] = m;
    if (bad) sm_bad = 1;
    __syncthreads();
    m = smf[0];
#pragma unroll
    for (int w = 1; w < kQuantThreads / 64; ++w) m = fmaxf(m, smf[w]);
    bad = sm_bad;

    // step = 2^(e-22) with m = f * 2^e, f in [0.5, 1)  ->  |q| <= 2^22  (2^14 for the two-slice mode: the top byte slice is then zero)
    int e = 0;
    float step = 1.0f;
    if (m > 0.f && !bad) {
        (void)frexpf(m, &e);
        int se = e - (d.mag_exp > 0 ? d.mag_exp : 22);
        se = se < -126 ? -126 : se;            // stay a normal float; tiny inputs just lose bits
        step = ldexpf(1.0f, se);
    }
    const float inv_step = 1.0f / step;        // exact: power of two

    // pass 2: q = rint(v / step), split into three signed bytes, write the MFMA B-operand layout
    long long local_sum = 0;
    uint4* const dst = (uint4*)(d.bq) + (size_t)tok * d.n_chunks * kSlices;     // token-major, pieces ordered by bq_piece()
    if (held) {
#pragma unroll
        for (int k = 0; k < kQuantHeld; ++k) {
            const int c = tid + k * kQuantThreads;
            if (c < d.n_chunks)
                local_sum += quantize_chunk16<STREAMED>(hv[k], inv_step, bad, dst + bq_piece(c, 0));
        }
    } else {
        for (int c = tid; c < d.n_chunks; c += kQuantThreads) {
            float v[16];
            load_chunk16(d, base, c, vec, v);
            local_sum += quantize_chunk16<STREAMED>(v, inv_step, bad, dst + bq_piece(c, 0));
        }
    }
    double s = (double)local_sum;               // |sum| < 2^39: exact
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if ((tid & 63) == 0) smd[wave] = s;
    __syncthreads();
    if (tid == 0) {
        QMeta mt;
        double tot = 0.0;
        for (int w = 0; w < kQuantThreads / 64; ++w) tot += smd[w];
        mt.two_step = bad ? (double)__builtin_nanf("") : 2.0 * (double)step;
        mt.neg_qs = -tot * (double)step;
        d.meta[tok] = mt;
    }
}

// The same for short vectors (at most 64 * H chunks): ONE WAVE per (vector, token), its chunks
// held in registers between the two passes, reductions by shuffles only -- no workgroup barrier,
// no LDS; a workgroup is four independent waves.  A launch of many short vectors is a chain of
// latencies, not a stream: the 8192 (layer, token) pairs of 1024 ranks of 1024 at batch 8 took
// 22 us as workgroups of 256 threads of which 64 had a chunk, three barriers each, and take 14 us
// this way (13 -> 9 us at batch 4).  Taken for vectors of up to 1024 elements (H = 1); with more
// chunks per lane (H = 2, 4: vectors of up to 4096) it measured the same as the workgroup kernel
// or slower.  Same arithmetic element for element: identical bytes and constants.
template <int H, bool STREAMED>
__global__ void __launch_bounds__(256)
quantize_wave_kernel(const QuantDesc* __restrict__ descs, QuantDesc single, int n_ops, int batch)
{
    const int lane = threadIdx.x & 63;
    const int task = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (task >= n_ops * batch) return;                      // whole waves leave; nothing below synchronises
    const int op = task / batch, tok = task - op * batch;
    const QuantDesc d = descs ? descs[op] : single;
    const int64_t base = (int64_t)tok * d.x_stride;
    const int esz = d.dtype == NQ_F32 ? 4 : 2;
    const bool vec = (((size_t)d.x_stride * esz) & 15) == 0;

    float hv[H][16];
    float m = 0.f;
    int bad = 0;
#pragma unroll
    for (int k = 0; k < H; ++k) {
        // (a lane past the end re-reads the vector's first chunk: no branch around the loads, and
        // the maximum does not change)
        const int c = lane + 64 * k;
        load_chunk16(d, base, c < d.n_chunks ? c : 0, vec, hv[k]);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float a = fabsf(hv[k][i]);
            if (!(a <= 3.0e38f)) bad = 1;
            m = fmaxf(m, a);
        }
    }
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    bad = __builtin_amdgcn_ballot_w64(bad != 0) != 0;

    int e = 0;
    float step = 1.0f;
    if (m > 0.f && !bad) {
        (void)frexpf(m, &e);
        int se = e - (d.mag_exp > 0 ? d.mag_exp : 22);
        se = se < -126 ? -126 : se;
        step = ldexpf(1.0f, se);
    }
    const float inv_step = 1.0f / step;

    long long local_sum = 0;
    uint4* const dst = (uint4*)(d.bq) + (size_t)tok * d.n_chunks * kSlices;
#pragma unroll
    for (int k = 0; k < H; ++k) {
        const int c = lane + 64 * k;
        if (c < d.n_chunks) local_sum += quantize_chunk16<STREAMED>(hv[k], inv_step, bad != 0, dst + bq_piece(c, 0));
    }
    double sum = (double)local_sum;
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) {
        QMeta mt;
        mt.two_step = bad ? (double)__builtin_nanf("") : 2.0 * (double)step;
        mt.neg_qs = -sum * (double)step;
        d.meta[tok] = mt;
    }
}

// max_chunks: the largest n_chunks among the launch's vectors
int launch_quantize(const QuantDesc* d_descs, const QuantDesc& single, int n_ops, int max_chunks, int batch,
                    hipStream_t s)
{
    const bool no_wave = opt_flag(OPT_NO_QUANT_WAVE);
    // several short vectors: one wave each (a lone short vector keeps the workgroup kernel, whose
    // threads share it)
    if (!no_wave && max_chunks <= 64 && (size_t)n_ops * batch >= 64) {
        const dim3 wgrid((unsigned)(((size_t)n_ops * batch + 3) / 4));
#define NQ_LAUNCH_QWAVE(H)                                                                              \
    do {                                                                                                \
        if (batch <= 5) NQ_LAUNCH((quantize_wave_kernel<H, true>), wgrid, dim3(256), 0, s, d_descs, single, n_ops, batch); \
        else NQ_LAUNCH((quantize_wave_kernel<H, false>), wgrid, dim3(256), 0, s, d_descs, single, n_ops, batch);           \
    } while (0)
        NQ_LAUNCH_QWAVE(1);
#undef NQ_LAUNCH_QWAVE
        NQ_HIP(hipGetLastError());
        return NQ_OK;
    }
    const dim3 grid(n_ops, batch);
#define NQ_LAUNCH_QUANT(T)                                                                              \
    do {                                                                                                \
        if (batch <= 5) NQ_LAUNCH((quantize_kernel<T, true>), grid, dim3(T), 0, s, d_descs, single, batch); \
        else NQ_LAUNCH((quantize_kernel<T, false>), grid, dim3(T), 0, s, d_descs, single, batch);           \
    } while (0)
    if (max_chunks <= 256 * kQuantHeld) NQ_LAUNCH_QUANT(256);
    else if (max_chunks <= 512 * kQuantHeld) NQ_LAUNCH_QUANT(512);
    else NQ_LAUNCH_QUANT(1024);
#undef NQ_LAUNCH_QUANT
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// ---------------------------------------------------------------------------------------------
// sign + pack on the device (Algorithm 1, PackBinary; Fig. 2(c)): latent matrix [rows][cols] ->
// canonical words [rows][ceil(cols / 32)].  One wave per 64 consecutive columns of a row: the
// wave-wide ballot of "value >= 0" IS two packed words.  bit = 1 iff value >= 0 (both zeros -> +1);
// a NaN, or an int8 other than +-1, packs as bit 0 and is counted in *invalid.
// grid = (rows, ceil(cols / 256)), block = 256 (four waves, one 64-column chunk each)
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
pack_signs_kernel(const void* __restrict__ signs, int dtype, int64_t rows, int64_t cols, int64_t wpr,
                  uint32_t* __restrict__ words, int* __restrict__ invalid)
{
    const int lane = threadIdx.x & 63;
    const int64_t chunk = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);       // 64-column chunk of the row
    const int64_t row = blockIdx.x;
    const int64_t col = chunk * 64 + lane;
    if (chunk * 64 >= cols) return;
    bool plus = false, bad = false;
    if (col < cols) {
        const int64_t idx = row * cols + col;
        if (dtype == NQ_I8) {
            const int8_t v = ((const int8_t*)signs)[idx];
            plus = v == 1;
            bad = v != 1 && v != -1;
        } else {
            const float v = load_as_float(signs, dtype, idx);
            plus = v >= 0.0f;
            bad = v != v;
        }
    }
    const unsigned long long mask = __ballot(plus);
    if (bad && invalid) atomicAdd(invalid, 1);
    if (lane == 0) {
        words[row * wpr + chunk * 2] = (uint32_t)mask;
        if (chunk * 2 + 1 < wpr) words[row * wpr + chunk * 2 + 1] = (uint32_t)(mask >> 32);
    }
}

int launch_pack_signs(const void* d_signs, int dtype, int64_t rows, int64_t cols, uint32_t* d_words, int* d_invalid,
                      hipStream_t s)
{
    const int64_t wpr = (cols + 31) / 32;
    const int64_t chunks = (cols + 63) / 64;
    hipLaunchKernelGGL(pack_signs_kernel, dim3((unsigned)rows, (unsigned)((chunks + 3) / 4)), dim3(256), 0, s, d_signs,
                       dtype, rows, cols, wpr, d_words, d_invalid);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// ---------------------------------------------------------------------------------------------
// streaming sign-matrix x fixed-point-vector kernels (steps a2 and a4, with a5 fused in stage 2)
//   NB : number of 16-column groups of the B operand (1: batch <= 5, 2: batch 6..8)
//   D  : software prefetch ring (tiles per wave; D-1 stay in flight while one is consumed)
// Three schedules over the same tiles:
//   stage_stream_kernel : one wave per work item.  An item is a row block, or a run of a few
//       consecutive short ones of one op; their tiles are contiguous in memory, so the prefetch
//       ring keeps running across block boundaries and only the accumulators are flushed there.
//       For short reductions.
//   stage_split_kernel<W> : W waves of one workgroup interleave the 64-column steps of ONE row
//       block and are summed through LDS.  For long reductions, and for launches with too few row
//       blocks to fill the chip.
//   stage_shared_kernel : the waves of a workgroup take row blocks of one op and share its quantised input
//       through LDS (further down).  For two column groups in launches that fill the chip.
// In all of them a grid as large as the item list makes the hardware workgroup dispatcher the
// work queue (the list is sorted longest first).
// ---------------------------------------------------------------------------------------------
#ifndef NQ_STAGE_WAVES
#define NQ_STAGE_WAVES 5
#endif
// Pointers that come out of a descriptor in memory are generic to the compiler; accesses through
// them would be flat instructions, which count on two wait counters at once and make every later
// wait a "wait for everything".  These casts name the address space: global for vector accesses,
// constant for wave-uniform reads (scalar loads, which the vector-memory counter does not see).
typedef const __attribute__((address_space(1))) uint16_t* gptr_u16;
typedef const __attribute__((address_space(4))) QMeta* cptr_meta;

// Byte offset, inside an op's quantised input, of the 16 bytes lane (g, n) feeds to the MFMA as
// rows 16g..16g+15 of column n of column group cg, at step 0.  The input is token-major
// ([token][step][slice][chunk of the step][16 bytes], a step = kBqStepBytes); column n of a group is
// slice n % 3 of the group's token n / 3.  Lanes of unused columns (n = 15, or a token beyond the
// batch) re-read token 0: their result columns are never looked at.
__device__ __forceinline__ uint32_t bq_lane_offset(int cg, int g, int n, int batch, int nst)
{
    int tok = 5 * cg + n / 3;
    const int slice = n % 3;
    if (n >= 15 || tok >= batch) tok = 0;
    return (uint32_t)tok * ((uint32_t)nst * kBqStepBytes) + (uint32_t)(bq_piece(g, slice) * 16);
}

struct EpilogueArgs {
    const QMeta* meta;
    const uint16_t* out_scale;
    void* out;
    int M, out_stride, out_dtype;
};

// LDS ints one wave needs for the epilogue: 16 columns x 64 rows
// ints between the 16 columns of a wave's epilogue region: the 64 rows of a half plus 4 -- with 64 (256 bytes, once round
// the LDS banks) the 16-byte writes of the up to 15 lanes that hold the columns of one row group all fell on the same
// banks (counters on the batch-8 kernels: 59-65 % of the LDS's active cycles were bank conflicts)
constexpr int kEpiCol = 68;
constexpr int kEpiRegion = 16 * kEpiCol;
// LDS ints a wave of stage_selfq_kernel needs: its quantised share (16 steps of 192 bytes per chunk
// a lane holds), later its epilogue region
constexpr int selfq_region_ints(int chunks_per_lane) { return chunks_per_lane * 16 * 192 / 4 > kEpiRegion ? chunks_per_lane * 16 * 192 / 4 : kEpiRegion; }
// most row blocks an item of the stream kernel may chain
constexpr int kStreamMaxRbs = 8;

// raw accumulators -> LDS [col][row] -> one thread per (token, row): undo the plane weights,
// join the three byte slices, apply 2*sum(b q) - sum(q), the step and the output scale.
// The 128 rows x (3 columns per token) results pass through LDS in pieces of 64 rows (four bit planes) x one
// column group, so that the LDS a wave holds (and with it the number of resident waves) does not
// grow with the batch.
// W = 1: `lds` is this wave's private region and only the wave synchronises;
// W > 1: `lds` is the workgroup's buffer of W regions and the partial sums of the W waves are added.
// DEFER: the results go to `lds_out[128 * batch]` (token-major), not yet multiplied by the output
// scale, instead of global memory; the stream kernel scales and stores them after the item's last
// row block.  In the middle of the stream the epilogue must issue no vector memory operation: a
// pending store would force every later wait on the prefetch ring down to "wait for everything"
// (loads and stores share one in-order counter only among their own kind), and waiting for a
// freshly issued load means waiting for the whole ring issued before it.  The per-token constants
// come through scalar loads, which that counter does not see.
// `pre_scale` (or nullptr): the output scales (fp16 bits) of this lane's two rows (row lane of each
// half), fetched by the caller ahead of time and converted only here, so that nothing waits for them early; `own_meta` (or nullptr): the constants of token 0 when the
// caller has just computed them itself (batch 1).  Both only shorten the chain of dependent memory
// round trips of a launch that is bound by latency.
// SL: byte slices (MFMA columns) per token: 3, five tokens per column group; or 2 (16-bit fixed point, the middle and low
// slices), eight tokens in the one group.
template <int NB, int W, bool DEFER, int SL = 3>
__device__ __forceinline__ void stage_epilogue(const v4i (&acc)[NB][8], int* lds, int wave, int lane, int batch,
                                               int rb, const EpilogueArgs& e, float* lds_out,
                                               const uint16_t* pre_scale = nullptr, const QMeta* own_meta = nullptr,
                                               int region = kEpiRegion, bool meta_is_partial = false)
{
    // `region`: ints between the LDS regions of the W waves (their first kEpiRegion ints are used here).
    // meta_is_partial: own_meta->neg_qs is this wave's share of -sum(q) step; the shares of the W
    // waves, which the caller has put into the (otherwise unused) column 15 of their regions, are added.
    const int g = lane >> 4, n = lane & 15;
    int* my_lds = (W == 1) ? lds : lds + wave * region;
    const cptr_meta meta = (cptr_meta)e.meta;
#pragma unroll
    for (int cg = 0; cg < NB; ++cg) {
        constexpr int kTokPerGroup = SL == 3 ? 5 : 8;
        static_assert(SL == 3 || NB == 1, "two slices: one column group");
        const int tg = batch - kTokPerGroup * cg < kTokPerGroup ? batch - kTokPerGroup * cg : kTokPerGroup;      // tokens in this column group
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            // accumulator layout of the 16x16 result: lane (g, n), register v <-> D[row 4g+v][col n];
            // the four registers of a plane are four consecutive rows: one 16-byte LDS write per plane
            if (n < SL * tg) {
                v4i* dst = (v4i*)(my_lds + n * kEpiCol + 4 * g);
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    // plane 7 (the int8 sign bit) holds -128 * sum: stored negated, so that every plane p reads 2^p * sum
                    const v4i a = acc[cg][4 * hf + p];
                    dst[4 * p] = (4 * hf + p == 7) ? -a : a;                       // rows 16p + 4g .. +3 of the half
                }
            }
            if (W == 1) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            } else {
                __syncthreads();
            }
            // one lane per row of the half; the token is the same for the whole wave
            const int row = lane;
            const int r128 = 64 * hf + row;
            const int grow = rb * kTileRows + r128;
            const int neg_p = -(4 * hf + (row >> 4));                 // this row's sums carry the weight 2^p of its plane
            float oscale = 1.0f;
            if (pre_scale) oscale = e.out_scale ? half_bits_to_float(pre_scale[hf]) : 1.0f;
            else if (!DEFER && e.out_scale && grow < e.M) oscale = half_bits_to_float(((gptr_u16)e.out_scale)[grow]);
            auto one_token = [&](int tl) {
                int h = 0, m = 0, l = 0;
#pragma unroll
                for (int w = 0; w < W; ++w) {
                    const int* q = lds + w * region + (SL * tl) * kEpiCol + row;
                    if (SL == 3) {
                        h += q[0];
                        m += q[kEpiCol];
                        l += q[2 * kEpiCol];
                    } else {
                        m += q[0];
                        l += q[kEpiCol];
                    }
                }
                // sum_n b_n q_n = (65536 h + 256 m + l) * 2^-p: the raw sums are below 2^30, so
                // every step is exact in fp64, and the plane's weight rides on the token's step
                const double raw = fma((double)h, 65536.0, fma((double)m, 256.0, (double)l));
                const int tok = kTokPerGroup * cg + tl;
                const double two_step = own_meta ? own_meta->two_step : meta[tok].two_step;
                double neg_qs = own_meta ? own_meta->neg_qs : meta[tok].neg_qs;
                if (own_meta && meta_is_partial && W > 1) {
                    neg_qs = 0.0;
#pragma unroll
                    for (int w = 0; w < W; ++w) neg_qs += *(const double*)(lds + w * region + 15 * kEpiCol);
                }
                const double val = fma(raw, __builtin_ldexp(two_step, neg_p), neg_qs);     // exact
                // z is rounded to fp32 here and multiplied by the output scale in fp32 -- by the flush for deferred
                // results, below for the others: the same two roundings on every path, so that the bits of y do not
                // depend on the schedule
                if (DEFER) {
                    lds_out[tok * kTileRows + r128] = (float)val;       // scaled by s_out when flushed
                } else if (grow < e.M) {
                    store_out(e.out, e.out_dtype, (size_t)tok * e.out_stride + grow, (float)val * oscale, e.out_scale != nullptr);
                }
            };
            for (int tl = wave; tl < tg; tl += W) one_token(tl);
            if (W == 1) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_wave_barrier();
            } else {
                __syncthreads();
            }
        }
    }
}

// End of an item of a streaming wave: the deferred results of its n_rb row blocks x batch tokens x
// 128 rows are scaled and stored.  The output scales of the item's rows (contiguous fp16, 16-byte
// loads of 8; the array is padded to whole row blocks) first go to the wave's now idle epilogue
// region `lds` as floats.
__device__ __forceinline__ void stream_flush(int* lds, const float* lds_out, int lane, int rb0, int n_rb, int batch,
                                             const EpilogueArgs& ea)
{
    float* lds_sc = (float*)lds;
    static_assert(kStreamMaxRbs * kTileRows <= kEpiRegion, "scales of an item must fit the epilogue region");
#pragma unroll
    for (int h = 0; h < kStreamMaxRbs * kTileRows / 512; ++h) {
        const int r0 = 512 * h + 8 * lane;
        if (r0 < n_rb * kTileRows) {
            float f[8];
            if (ea.out_scale) {
                const v4u raw = load_global_v4u((const char*)ea.out_scale, (uint32_t)((rb0 * kTileRows + r0) * 2));
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    f[2 * i] = half_bits_to_float((uint16_t)(raw[i] & 0xffffu));
                    f[2 * i + 1] = half_bits_to_float((uint16_t)(raw[i] >> 16));
                }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) f[i] = 1.0f;
            }
            *(v4f*)(lds_sc + r0) = v4f{f[0], f[1], f[2], f[3]};
            *(v4f*)(lds_sc + r0 + 4) = v4f{f[4], f[5], f[6], f[7]};
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    // one loop nest per output type (the type is the same for the whole item): a lane keeps its row
    // of each half of a row block and walks the tokens, so that an element costs one LDS read, one
    // multiplication and one store
    auto store_all = [&](auto store) {
        for (int u = 0; u < n_rb; ++u) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int row = 64 * hf + lane;
                const int grow = (rb0 + u) * kTileRows + row;
                if (grow >= ea.M) continue;
                const float sc = lds_sc[u * kTileRows + row];
                const float* src = lds_out + u * (kTileRows * batch) + row;
                size_t idx = (size_t)grow;
                for (int tok = 0; tok < batch; ++tok, idx += (size_t)ea.out_stride) store(idx, src[tok * kTileRows] * sc);
            }
        }
    };
    typedef __attribute__((address_space(1))) float* gptr_f32;
    typedef __attribute__((address_space(1))) uint16_t* gptr_o16;
    // (a final output -- the stage with output scales -- is stored non-temporal, see store_out)
    if (ea.out_dtype == NQ_F32) {
        if (ea.out_scale) store_all([&](size_t i, float v) { __builtin_nontemporal_store(v, (gptr_f32)ea.out + i); });
        else store_all([&](size_t i, float v) { ((gptr_f32)ea.out)[i] = v; });
    } else if (ea.out_dtype == NQ_BF16) {
        store_all([&](size_t i, float v) { __builtin_nontemporal_store(float_to_bf16_bits(v), (gptr_o16)ea.out + i); });
    } else {
        store_all([&](size_t i, float v) { __builtin_nontemporal_store(float_to_f16_bits(v), (gptr_o16)ea.out + i); });
    }
}

#define NQ_LOAD_ITEM()                                                                             \
    const uint32_t* tiles;                                                                         \
    const uint8_t* bq;                                                                             \
    int nst, rb0, n_rb;                                                                            \
    EpilogueArgs ea;                                                                               \
    if (items) {                                                                                   \
        const WorkItem* e = items + it;                                                            \
        tiles = e->tiles; bq = e->bq; nst = e->n_steps; rb0 = e->rb; n_rb = e->n_rb;               \
        const StageDesc* dp = descs + e->op;                                                       \
        ea.meta = dp->meta; ea.out_scale = dp->out_scale; ea.out = dp->out;                        \
        ea.M = dp->M; ea.out_stride = dp->out_stride; ea.out_dtype = dp->out_dtype;                \
    } else {                                                                                       \
        nst = single.n_steps;                                                                      \
        rb0 = it * rbs_per_item;                                                                   \
        const int total_rb = (single.M + kTileRows - 1) / kTileRows;                               \
        n_rb = total_rb - rb0 < rbs_per_item ? total_rb - rb0 : rbs_per_item;                      \
        tiles = single.tiles + (size_t)rb0 * nst * kTileWords;                                     \
        bq = single.bq;                                                                            \
        ea.meta = single.meta; ea.out_scale = single.out_scale; ea.out = single.out;               \
        ea.M = single.M; ea.out_stride = single.out_stride; ea.out_dtype = single.out_dtype;       \
    }

template <int NB, int D>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(NB == 1 ? NQ_STAGE_WAVES : 2, 8)))
stage_stream_kernel(const StageDesc* __restrict__ descs, StageDesc single, const WorkItem* __restrict__ items,
                    int n_items, int rbs_per_item, int batch)
{
    extern __shared__ int lds[];
    const int lane = threadIdx.x;
    const int g = lane >> 4, n = lane & 15;
    float* lds_out = (float*)(lds + kEpiRegion);            // [rbs of the item][batch][128 rows]
    for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
        // descriptor fields are wave-uniform (scalar loads); what the first tile load depends on
        // comes from the work item alone
        NQ_LOAD_ITEM()
        // 32-bit byte offsets from the (scalar) base pointers; a tile array is at most 512 MiB
        const char* a_base = (const char*)tiles;
        const char* b_base = (const char*)bq;
        uint32_t a_off = (uint32_t)(lane * 16);
        uint32_t b_lane[NB];
#pragma unroll
        for (int cg = 0; cg < NB; ++cg) b_lane[cg] = bq_lane_offset(cg, g, n, batch, nst);
        const uint32_t b_inc = kBqStepBytes;
        int b_step = 0;                                    // step (inside its row block) of the next tile to fetch

        v4u wbuf[D];
        v4u bbuf[D][NB];
        // fetch the next tile of the item's stream into slot k; the activation offset wraps at a
        // row-block boundary (scalar arithmetic), the tile offset just runs on
#define NQ_ISSUE(k)                                                              \
    do {                                                                         \
        wbuf[k] = load_tile_words(a_base, a_off);                                \
        a_off += 1024;                                                           \
        _Pragma("unroll") for (int cg = 0; cg < NB; ++cg)                        \
            bbuf[k][cg] = load_global_v4u(b_base, b_lane[cg] + (uint32_t)b_step * b_inc); \
        b_step = (b_step + 1 == nst) ? 0 : b_step + 1;                           \
    } while (0)

        // nst is a multiple of D (the tile layout pads the reduction to 4 steps), so every row
        // block starts in slot 0 and the ring never needs a partial group
#pragma unroll
        for (int k = 0; k < D; ++k) {
            NQ_ISSUE(k);
            __builtin_amdgcn_sched_barrier(0);             // same issue order as inside the loop
        }
        const int groups = nst / D;
        // all row blocks but the last: results deferred through LDS
        for (int u = 0; u + 1 < n_rb; ++u) {
            v4i acc[NB][8];
#pragma unroll
            for (int cg = 0; cg < NB; ++cg)
#pragma unroll
                for (int p = 0; p < 8; ++p) acc[cg][p] = v4i{0, 0, 0, 0};
            for (int gi = 0; gi < groups; ++gi) {
#pragma unroll
                for (int k = 0; k < D; ++k) {
                    mac_tile<NB>(acc, wbuf[k], bbuf[k]);
                    NQ_ISSUE(k);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            stage_epilogue<NB, 1, true>(acc, lds, 0, lane, batch, rb0 + u, ea,
                                        lds_out + u * (kTileRows * batch));
        }
        // the last one must not fetch past its own tiles; the ring is empty after it, so its
        // results are scaled and stored straight from the epilogue
        {
            v4i acc[NB][8];
#pragma unroll
            for (int cg = 0; cg < NB; ++cg)
#pragma unroll
                for (int p = 0; p < 8; ++p) acc[cg][p] = v4i{0, 0, 0, 0};
            for (int gi = 0; gi < groups - 1; ++gi) {
#pragma unroll
                for (int k = 0; k < D; ++k) {
                    mac_tile<NB>(acc, wbuf[k], bbuf[k]);
                    NQ_ISSUE(k);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int k = 0; k < D; ++k) {
                mac_tile<NB>(acc, wbuf[k], bbuf[k]);
                __builtin_amdgcn_sched_barrier(0);
            }
            stage_epilogue<NB, 1, false>(acc, lds, 0, lane, batch, rb0 + n_rb - 1, ea, nullptr);
        }
#undef NQ_ISSUE
        if (n_rb > 1) stream_flush(lds, lds_out, lane, rb0, n_rb - 1, batch, ea);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
    }
}

template <int NB, int W, int D>
__global__ void __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(NB == 1 ? NQ_STAGE_WAVES : 2, 8)))
stage_split_kernel(const StageDesc* __restrict__ descs, StageDesc single, const WorkItem* __restrict__ items,
                   int n_items, int batch)
{
    extern __shared__ int lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, n = lane & 15;
    constexpr int rbs_per_item = 1;
    const int st0 = wave;

    for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
        NQ_LOAD_ITEM()
        (void)n_rb;
        const int cnt = (nst - st0 + W - 1) / W;         // steps this wave performs (may be <= 0)
        // (a wave with no step of its own, possible when W > nst, aims its unused prefetches at step 0)
        const int stf = cnt > 0 ? st0 : 0;
        const char* a_base = (const char*)tiles;
        const char* b_base = (const char*)bq;
        uint32_t a_off = (uint32_t)(stf * 1024 + lane * 16);
        uint32_t b_off[NB];
#pragma unroll
        for (int cg = 0; cg < NB; ++cg) b_off[cg] = (uint32_t)stf * kBqStepBytes + bq_lane_offset(cg, g, n, batch, nst);
        const uint32_t b_inc = (uint32_t)W * kBqStepBytes;

        v4i acc[NB][8];
#pragma unroll
        for (int cg = 0; cg < NB; ++cg)
#pragma unroll
            for (int p = 0; p < 8; ++p) acc[cg][p] = v4i{0, 0, 0, 0};

        v4u wbuf[D];
        v4u bbuf[D][NB];
#define NQ_ISSUE(k)                                                              \
    do {                                                                         \
        wbuf[k] = load_tile_words(a_base, a_off);                                \
        a_off += W * 1024;                                                       \
        _Pragma("unroll") for (int cg = 0; cg < NB; ++cg) {                      \
            bbuf[k][cg] = load_global_v4u(b_base, b_off[cg]);                    \
            b_off[cg] += b_inc;                                                  \
        }                                                                        \
    } while (0)

        // prologue: D tiles in flight.  Issued unconditionally and branch-free (a short share
        // re-reads its last tile into the unused slots) so that the number of outstanding loads
        // at the loop head is the same on every path and the waits inside the loop stay partial.
        {
#pragma unroll
            for (int k = 0; k < D; ++k) {
                const int kk = k < cnt ? k : (cnt > 0 ? cnt - 1 : 0);
                wbuf[k] = load_tile_words(a_base, a_off + (uint32_t)kk * (W * 1024));
#pragma unroll
                for (int cg = 0; cg < NB; ++cg) bbuf[k][cg] = load_global_v4u(b_base, b_off[cg] + (uint32_t)kk * b_inc);
            }
            a_off += D * W * 1024;
#pragma unroll
            for (int cg = 0; cg < NB; ++cg) b_off[cg] += D * b_inc;
        }
        int i0 = 0;
        // steady state: compute on a slot, then refill it; the scheduling barriers keep the
        // loads interleaved with the compute (D-1 tiles stay in flight) instead of bunched
        for (; i0 + 2 * D <= cnt; i0 += D) {
#pragma unroll
            for (int k = 0; k < D; ++k) {
                mac_tile<NB>(acc, wbuf[k], bbuf[k]);
                NQ_ISSUE(k);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // last D..2D-1 steps: refill only while tiles remain
#pragma unroll
        for (int k = 0; k < D; ++k) {
            if (i0 + k < cnt) {
                mac_tile<NB>(acc, wbuf[k], bbuf[k]);
                if (i0 + k + D < cnt) NQ_ISSUE(k);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int k = 0; k < D; ++k) {
            if (i0 + D + k < cnt) {
                mac_tile<NB>(acc, wbuf[k], bbuf[k]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#undef NQ_ISSUE
        stage_epilogue<NB, W, false>(acc, lds, wave, lane, batch, rb0, ea, nullptr);
    }
}
// ---------------------------------------------------------------------------------------------
// Third schedule, for batch 6..8 (two column groups) and the long reductions of batch 4..5, in
// launches that fill the chip: the W =
// kShareWaves waves of a workgroup take row blocks of ONE op and share its quantised input through
// LDS.  With the B operand out of the registers (and off the vector-memory counter, which returns
// loads in order) a wave affords a ring of eight tiles although the 64 accumulator registers
// leave room for two waves per SIMD only; and the input is fetched from L2 once per W or more
// row blocks instead of once per row block.  W = 4, so that TWO workgroups share a CU and one
// streams while the other stages its input, waits at a barrier or flushes its results: with W = 8
// (one workgroup per CU, nothing to overlap with) the 1024-layer pool of 4096x4096 r=1024 layers
// took 377 us per step at batch 8, with W = 4 it takes 349 (stage 1 139 -> 129, stage 2 188 -> 168).
//   - the input is staged in chunks of 8 steps (one pass over the ring), double buffered; every
//     wave fetches 1/W of the next chunk at the start of a pass and writes it to LDS at the end
//     (by then those loads are the oldest outstanding ones); one barrier per pass;
//   - wave w owns `per` = ceil(n_rb / W) consecutive row blocks of the item (their tiles are
//     contiguous, the ring runs on across them); results are deferred through LDS as in the
//     stream kernel;
//   - a reduction that is not a multiple of 8 steps ends in half a pass, so such ops get one row
//     block per wave (the host sees to that);
//   - refills past the wave's last tile re-read that tile, and a wave with fewer row blocks than
//     its siblings keeps multiplying that tile without storing anything: no branches around
//     loads, the wait counts stay exact.
// LDS: [2][batch][kShareTokStride] input | [W][kEpiRegion] epilogue | [W][per_max][128 * batch] results.
// ---------------------------------------------------------------------------------------------
constexpr int kShareChunk = 8;
// bytes between tokens of a staged chunk; = 48 mod 256, which spreads the 15 (token, slice)
// operands of a 16-lane group over all LDS banks
constexpr int kShareTokStride = kShareChunk * (int)kBqStepBytes + 48;
static_assert(kShareTokStride % 256 == 48, "bank spread");

// RESIDENT: for reductions of at most 16 steps the whole quantised input (two chunks) is staged once
// per item and stays in its two buffers; the row blocks then need neither refills nor barriers, and
// the waves drift apart freely.
// SL = 2: the input is 16-bit fixed point (slices 1 and 2 of the three-slice layout, slice 0 is zero and is not fed to the
// matrix cores): column n of the one group is slice 1 + n % 2 of token n / 2.
template <int NB, bool RESIDENT, int SL = 3>
__global__ void __launch_bounds__(64 * kShareWaves) __attribute__((amdgpu_waves_per_eu(NB == 2 ? 2 : 3, NB == 2 ? 2 : 8)))
stage_shared_kernel(const StageDesc* __restrict__ descs, const WorkItem* __restrict__ items, int n_items, int per_max,
                    int batch)
{
    extern __shared__ int lds[];
    constexpr int W = kShareWaves;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int buf_bytes = batch * kShareTokStride;
    char* const lds_b = (char*)lds;
    int* const lds_epi = (int*)(lds_b + 2 * buf_bytes) + wave * kEpiRegion;
    float* const lds_out = (float*)((int*)(lds_b + 2 * buf_bytes) + W * kEpiRegion) + wave * (per_max * kTileRows * batch);

    // this lane's operand inside a staged chunk (step 0).  An unused column re-reads the group's LAST used one: the same
    // address, which the LDS broadcasts -- token 0's pieces would be other addresses on the banks of the octet's own
    // operands (the LDS serves 128 bytes, eight lanes of a 16-byte read, per cycle).  (The conflict counter of the
    // batch-8 launches falls by a sixth with it; their duration does not change.)
    uint32_t b_lds[NB];
#pragma unroll
    for (int cg = 0; cg < NB; ++cg) {
        constexpr int kTokPerGroup = SL == 3 ? 5 : 8;
        int used = SL * (batch - kTokPerGroup * cg);                    // columns of this group that carry a token
        used = used > SL * kTokPerGroup ? SL * kTokPerGroup : (used < 1 ? 1 : used);
        const int col = n < used ? n : used - 1;
        int tok = kTokPerGroup * cg + col / SL;
        const int slice = SL == 3 ? col % 3 : 1 + col % 2;
        if (tok >= batch) tok = 0;                                      // (a group without tokens: never used)
        b_lds[cg] = (uint32_t)(tok * kShareTokStride + (g * kSlices + slice) * 16);
    }
    // this thread's share of a chunk: 16-byte pieces id = i * 512 + tid < batch * 96 (i < 2);
    // piece id -> token id / 96, offset (id % 96) * 16 inside the token's chunk.  A thread without
    // a piece copies piece 0 as well (same bytes to the same place), which keeps the copy free of
    // branches and the wait counts the same on every path.
    constexpr int kPiecesPerTok = kShareChunk * (int)kBqStepBytes / 16;        // 96
    constexpr int kShare = (8 * kPiecesPerTok + 64 * kShareWaves - 1) / (64 * kShareWaves);
    static_assert(kShare * 64 * kShareWaves >= 8 * kPiecesPerTok, "a chunk of 8 tokens in kShare pieces per thread");
    uint32_t sh_src[kShare], sh_dst[kShare];
#pragma unroll
    for (int i = 0; i < kShare; ++i) {
        const int id = i * (64 * W) + tid;
        const int idc = id < batch * kPiecesPerTok ? id : 0;
        const int tok = idc / kPiecesPerTok, piece = idc - tok * kPiecesPerTok;
        sh_src[i] = (uint32_t)(piece * 16);                                   // + tok * (one token's bytes), per item
        // in LDS the three slices of a chunk are adjacent (bank spread of the operand reads): piece
        // (step, slice, g) of the global order goes to (step, g, slice)
        const int st = piece / 12, sl = piece % 12 / 4, gg = piece % 4;
        sh_dst[i] = (uint32_t)(tok * kShareTokStride + (st * 12 + gg * kSlices + sl) * 16);
    }

    for (int it = blockIdx.x; it < n_items; it += gridDim.x) {
        const WorkItem* e = items + it;
        const int nst = e->n_steps, n_rb = e->n_rb, rb_first = e->rb;
        const char* const b_base = (const char*)e->bq;
        const StageDesc* dp = descs + e->op;
        EpilogueArgs ea;
        ea.meta = dp->meta; ea.out_scale = dp->out_scale; ea.out = dp->out;
        ea.M = dp->M; ea.out_stride = dp->out_stride; ea.out_dtype = dp->out_dtype;
        const int per = (n_rb + W - 1) / W;
        const int my0 = wave * per;
        const int my_n = n_rb - my0 < per ? (n_rb - my0 > 0 ? n_rb - my0 : 0) : per;
        const int passes = nst >> 3;                                    // full passes per row block
        const int chunks = (nst + kShareChunk - 1) / kShareChunk;       // passes + the half pass, if any
        const uint32_t tok_bytes = (uint32_t)nst * kBqStepBytes;         // one token's quantised input
        uint32_t sh_off[kShare];
#pragma unroll
        for (int i = 0; i < kShare; ++i) sh_off[i] = (sh_dst[i] / kShareTokStride) * tok_bytes + sh_src[i];

        // the wave's tile stream (a wave without a row block aims at the item's first tile)
        const char* const a_base = (const char*)(e->tiles) + (size_t)(my_n > 0 ? my0 : 0) * nst * (kTileWords * 4);
        uint32_t a_off = (uint32_t)(lane * 16);
        const uint32_t a_last = (uint32_t)(((my_n > 0 ? my_n * nst : 1) - 1) * 1024 + lane * 16);
        v4u wbuf[8];
#define NQ_ISSUE(k)                                                              \
    do {                                                                         \
        wbuf[k] = load_tile_words(a_base, a_off);                                \
        a_off = a_off + 1024 < a_last ? a_off + 1024 : a_last;                   \
    } while (0)
        // this thread's share of chunk c (the half pass stages a whole chunk too: the quantised
        // input is padded to 4 steps and the allocation to more, see the workspace layout)
#define NQ_SHARE_LOAD(c)                                                         \
    _Pragma("unroll") for (int i = 0; i < kShare; ++i)                           \
        sh[i] = load_global_v4u(b_base, sh_off[i] + (uint32_t)((c) * kShareChunk) * kBqStepBytes)
#define NQ_SHARE_STORE(buf)                                                      \
    _Pragma("unroll") for (int i = 0; i < kShare; ++i)                           \
        *(v4u*)(lds_b + (buf) * buf_bytes + sh_dst[i]) = sh[i]
        v4u sh[kShare];

        __syncthreads();                                   // the previous item's readers are done with the buffers
        int round = 0;                                     // chunks consumed so far
        // The input (from L2) is requested BEFORE the ring's first tiles (from HBM): loads return
        // in order, so the staging and its barrier then run while the tiles are still on their way
        // instead of after the last of them has arrived (stage 2 of the 4096x4096 r=1024 pool at
        // batch 8: 175 -> 168 us).
        v4u sh1[kShare];
        NQ_SHARE_LOAD(0);
        if (RESIDENT) {
#pragma unroll
            for (int i = 0; i < kShare; ++i)
                sh1[i] = load_global_v4u(b_base, sh_off[i] + (uint32_t)((chunks > 1 ? 1 : 0) * kShareChunk) * kBqStepBytes);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            NQ_ISSUE(k);
            __builtin_amdgcn_sched_barrier(0);
        }
        NQ_SHARE_STORE(0);
        if (RESIDENT) {                                    // (a one-chunk input is copied twice: no branch around loads)
#pragma unroll
            for (int i = 0; i < kShare; ++i) *(v4u*)(lds_b + buf_bytes + sh_dst[i]) = sh1[i];
            __syncthreads();
        }

        // operands of step j of the current chunk
#define NQ_LDSB(dst, j)                                                          \
    _Pragma("unroll") for (int cg = 0; cg < NB; ++cg)                            \
        dst[cg] = *(const v4u*)(bb + b_lds[cg] + (j) * (int)kBqStepBytes)
        // `cnt` steps on ring slots 0.., operands prefetched one step ahead
#define NQ_PASS(cnt)                                                             \
    do {                                                                         \
        v4u bop[2][NB];                                                          \
        NQ_LDSB(bop[0], 0);                                                      \
        _Pragma("unroll") for (int k = 0; k < (cnt); ++k) {                      \
            if (k + 1 < (cnt)) NQ_LDSB(bop[(k + 1) & 1], k + 1);                 \
            mac_tile<NB>(acc, wbuf[k], bop[k & 1]);                              \
            NQ_ISSUE(k);                                                         \
            __builtin_amdgcn_sched_barrier(0);                                   \
        }                                                                        \
    } while (0)

        // one row block of this wave: full passes, then (HALF) the closing half pass
#define NQ_ROW_BLOCK(u, HALF)                                                    \
    do {                                                                         \
        v4i acc[NB][8];                                                          \
        _Pragma("unroll") for (int cg = 0; cg < NB; ++cg)                        \
            _Pragma("unroll") for (int p = 0; p < 8; ++p) acc[cg][p] = v4i{0, 0, 0, 0}; \
        if (RESIDENT) {                                                          \
            for (int c = 0; c < passes; ++c) {                                   \
                const char* const bb = lds_b + c * buf_bytes;                    \
                NQ_PASS(8);                                                      \
            }                                                                    \
            if (HALF) {                                                          \
                const char* const bb = lds_b + passes * buf_bytes;               \
                NQ_PASS(4);                                                      \
            }                                                                    \
        } else {                                                                 \
            for (int c = 0; c < passes; ++c, ++round) {                          \
                __syncthreads();         /* chunk c is in its buffer; the other buffer is free */ \
                const char* const bb = lds_b + (round & 1) * buf_bytes;          \
                NQ_SHARE_LOAD(c + 1 == chunks ? 0 : c + 1);                      \
                NQ_PASS(8);                                                      \
                NQ_SHARE_STORE((round & 1) ^ 1);                                 \
            }                                                                    \
            if (HALF) {                                                          \
                __syncthreads();                                                 \
                const char* const bb = lds_b + (round & 1) * buf_bytes;          \
                NQ_PASS(4);                                                      \
                ++round;                                                         \
            }                                                                    \
        }                                                                        \
        if ((u) < my_n)                                                          \
            stage_epilogue<NB, 1, true, SL>(acc, lds_epi, 0, lane, batch, rb_first + my0 + (u), ea, \
                                            lds_out + (u) * (kTileRows * batch)); \
    } while (0)

        if (nst & 4) {
            // the half pass leaves the ring out of phase: it must be the last thing the wave
            // computes, so such an item has one row block per wave
            NQ_ROW_BLOCK(0, true);
        } else {
            for (int u = 0; u < per; ++u) NQ_ROW_BLOCK(u, false);
        }
#undef NQ_ROW_BLOCK
#undef NQ_PASS
#undef NQ_LDSB
#undef NQ_SHARE_STORE
#undef NQ_SHARE_LOAD
#undef NQ_ISSUE
        if (my_n > 0) stream_flush(lds_epi, lds_out, lane, rb_first + my0, my_n, batch, ea);
    }
}

// ---------------------------------------------------------------------------------------------
// Batch 1: the stream / split schedules with the quantisation of the input done by the waves
// themselves, which removes the two quantisation launches of a step (19 of 205 us on the
// 1024-layer pool; 4 of a lone layer's dependent launch latencies become 2) and takes the B
// operand off the vector-memory path.
// A wave requests its first D tiles, reads the chunks of its OWN steps (wave, wave + W, ...), takes
// their maximum (with W = 4 the four waves exchange theirs through LDS: the step follows from the
// maximum of the whole vector), quantises its chunks into its LDS region in the layout of the
// global buffer, and streams its tiles with the B operand read from LDS one step ahead.  The
// sum of its quantised values goes through column 15 of its epilogue region to the wave that
// finishes the token.  After the wave's last step its region is reused for the epilogue.
// The arithmetic is that of quantize_kernel + stage_{stream,split}_kernel element for element.
// One item = one row block; W = 1 (short reductions) or 4 (long ones, split as in the split kernel).
// Only for shares of at most 16 steps per wave (reductions of up to 1024 elements with W = 1, 4096
// with W = 4): a lane then owns ONE chunk of 16 values, loaded once and kept in registers between
// the maximum and the quantisation, and the 3 KiB of quantised input fit the epilogue region.  With
// longer shares (chunks read twice, more LDS, fewer resident waves) the separate quantisation
// launch measured faster: 4096x8192 r=1024 164 vs 169 us per step of a 512-layer pool, 11008x4096
// r=1664 135 vs 143 us; the 1024-layer pool of 4096x4096 r=1024 layers gains 205 -> 191 us.
// LDS: [W][kEpiRegion] (+ W maxima and flags when W = 4).
// LIST: workgroup i takes items[i]; otherwise row block i of the one op in the kernel arguments q1 / s1.
// ---------------------------------------------------------------------------------------------
// C: chunks of 16 values a lane holds (1: shares of at most 16 steps; 2: up to 32, with one wave per
// row block only -- the quantised share then takes 6 KiB of LDS per wave instead of 3).
template <int W, int D, bool LIST, int C = 1>
__global__ void __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(C == 1 ? NQ_STAGE_WAVES : 4, 8)))
stage_selfq_kernel(const FusedItem* __restrict__ items, QuantDesc q1, StageDesc s1)
{
    static_assert(C == 1 || W == 1, "two chunks per lane only with one wave per row block");
    constexpr int region = selfq_region_ints(C);
    extern __shared__ int lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, n = lane & 15;
    int rb = blockIdx.x;
    QuantDesc qd = q1;
    StageDesc sd = s1;
    if (LIST) {
        const FusedItem* e = items + blockIdx.x;           // uniform address of a kernel argument: scalar loads
        rb = e->rb;
        qd = e->q;
        sd = e->s;
    }
    const int nst = sd.n_steps;
    char* const my_bq = (char*)(lds + wave * region);

    const int cnt = (nst - wave + W - 1) / W;              // steps of this wave (may be <= 0 when W > nst)
    const int stf = cnt > 0 ? wave : 0;
    const char* const a_base = (const char*)sd.tiles + (size_t)rb * nst * (kTileWords * 4);
    uint32_t a_off = (uint32_t)(stf * 1024 + lane * 16);

    // ---- the wave quantises the chunks of its own steps ----
    // lane j owns local chunk j = chunk j % 4 of the wave's step j / 4; the W waves' chunks
    // together cover the vector (chunks past its end read as zeros).  (Requesting the input ahead
    // of the tiles, so that the quantisation runs while the tiles are on their way, measured the same.)
    const int esz = qd.dtype == NQ_F32 ? 4 : 2;
    const bool vec = (((size_t)qd.x_stride * esz) & 15) == 0;
    const int n_own = 4 * cnt;                             // <= 64 C (the host checks the reduction length)
    float hv[C][16];
    float m = 0.f;
    int bad = 0;
    // (a lane beyond n_own reads a chunk of zeros or of another wave: harmless for the maximum)
    const int my_chunk = 4 * (wave + (lane >> 2) * W) + (lane & 3);     // the c-th chunk of a lane: + 64 c W

    v4u wbuf[D];
#pragma unroll
    for (int k = 0; k < D; ++k) {                          // branch-free: a short share re-reads its last tile
        const int kk = k < cnt ? k : (cnt > 0 ? cnt - 1 : 0);
        wbuf[k] = load_tile_words(a_base, a_off + (uint32_t)kk * (W * 1024));
    }
    a_off += D * W * 1024;
    uint16_t pre_scale[2];
    {
        const gptr_u16 sp = sd.out_scale ? (gptr_u16)sd.out_scale + rb * kTileRows : (gptr_u16)a_base;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) pre_scale[hf] = sp[64 * hf + lane];
    }
#pragma unroll
    for (int c = 0; c < C; ++c) load_chunk16(qd, 0, my_chunk + 64 * c * W, vec, hv[c]);
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float a = fabsf(hv[c][i]);
            if (!(a <= 3.0e38f)) bad = 1;
            m = fmaxf(m, a);
        }
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    bad = __builtin_amdgcn_ballot_w64(bad != 0) != 0;
    if (W > 1) {
        // the step follows from the maximum over the whole vector: one exchange between the waves
        float* const red_f = (float*)(lds + W * region);
        int* const red_bad = (int*)(red_f + W);
        if (lane == 0) {
            red_f[wave] = m;
            red_bad[wave] = bad;
        }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < W; ++w) {
            m = fmaxf(m, red_f[w]);
            bad |= red_bad[w];
        }
    }
    int ex = 0;
    float step = 1.0f;
    if (m > 0.f && !bad) {
        (void)frexpf(m, &ex);
        int se = ex - 22;
        se = se < -126 ? -126 : se;
        step = ldexpf(1.0f, se);
    }
    const float inv_step = 1.0f / step;
    long long local_sum = 0;
#pragma unroll
    for (int c = 0; c < C; ++c)
        if (lane + 64 * c < n_own)
            local_sum += quantize_chunk16(hv[c], inv_step, bad != 0, (uint4*)my_bq + bq_piece(lane + 64 * c, 0));
    double sum = (double)local_sum;
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    QMeta my_meta;
    my_meta.two_step = bad ? (double)__builtin_nanf("") : 2.0 * (double)step;
    my_meta.neg_qs = -sum * (double)step;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

    // ---- the reduction over this wave's steps ----
    const char* const b_lds = my_bq + bq_piece(g, n < 3 ? n : 0) * 16;      // token 0; unused columns re-read slice 0
    const int last = cnt > 0 ? cnt - 1 : 0;
    v4i acc[1][8];
#pragma unroll
    for (int p = 0; p < 8; ++p) acc[0][p] = v4i{0, 0, 0, 0};
#define NQ_ISSUE(k)                                                              \
    do {                                                                         \
        wbuf[k] = load_tile_words(a_base, a_off);                                \
        a_off += W * 1024;                                                       \
    } while (0)
#define NQ_LDSB(i) (*(const v4u*)(b_lds + ((i) < last ? (i) : last) * (int)kBqStepBytes))
    v4u bop[2][1];
    bop[0][0] = NQ_LDSB(0);
    int i0 = 0;
    for (; i0 + 2 * D <= cnt; i0 += D) {
#pragma unroll
        for (int k = 0; k < D; ++k) {
            bop[(k + 1) & 1][0] = NQ_LDSB(i0 + k + 1);
            mac_tile<1>(acc, wbuf[k], bop[k & 1]);
            NQ_ISSUE(k);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    static_assert(D % 2 == 0, "the operand double buffer is in phase at every pass over the ring");
#pragma unroll
    for (int k = 0; k < D; ++k) {
        if (i0 + k < cnt) {
            bop[(k + 1) & 1][0] = NQ_LDSB(i0 + k + 1);
            mac_tile<1>(acc, wbuf[k], bop[k & 1]);
            if (i0 + k + D < cnt) NQ_ISSUE(k);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int k = 0; k < D; ++k) {
        if (i0 + D + k < cnt) {
            bop[(k + 1) & 1][0] = NQ_LDSB(i0 + D + k + 1);
            mac_tile<1>(acc, wbuf[k], bop[k & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#undef NQ_LDSB
#undef NQ_ISSUE
    // the region changes hands: quantised input -> epilogue (wave-local, so no workgroup barrier)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    if (W > 1 && lane == 0) *(double*)(lds + wave * region + 15 * kEpiCol) = my_meta.neg_qs;
    EpilogueArgs ea;
    ea.meta = sd.meta; ea.out_scale = sd.out_scale; ea.out = sd.out;
    ea.M = sd.M; ea.out_stride = sd.out_stride; ea.out_dtype = sd.out_dtype;
    stage_epilogue<1, W, false>(acc, lds, wave, lane, 1, rb, ea, nullptr, pre_scale, &my_meta, region, W > 1);
}

// ---------------------------------------------------------------------------------------------
// Fourth schedule, for ONE layer on its own at batch 1 (nq_binlr_forward): a stage and the
// quantisation of its input in a single launch, so that a forward is two dependent launches
// instead of four -- a lone layer is bound by launch latency (about 4 us per dependent launch),
// not by bandwidth.  One workgroup of 16 waves per row block, as in the split kernel; every
// workgroup quantises the whole input vector for itself (one chunk of 16 values per thread, kept
// in registers between the max pass and the quantising pass) into LDS, in the layout of the
// global one, while its first tiles are already in flight; the MFMA B operands then come from
// LDS.  The arithmetic is that of quantize_kernel + stage_split_kernel, element for element, so
// the results are bit-identical.  Only for inputs of at most 16384 elements (fused_fits()).
// LDS: quantised input, overlaid after the reduction by [16][kEpiRegion] | scratch.
// ---------------------------------------------------------------------------------------------
constexpr int kFusedWaves = 16;
constexpr int kFusedScratchInts = 64;

__host__ __device__ inline size_t fused_lds_bytes(int nst)
{
    const size_t bq = (size_t)nst * kBqStepBytes, epi = (size_t)kFusedWaves * kEpiRegion * 4;
    return (bq > epi ? bq : epi) + kFusedScratchInts * 4;
}

// LIST: workgroup i takes items[i] (a row block of some op, with that op's descriptors inside: one
// fetch); otherwise row block i of the one op whose descriptors are the kernel arguments q1 / s1.
template <bool LIST>
__global__ void __launch_bounds__(64 * kFusedWaves) __attribute__((amdgpu_waves_per_eu(4, 8)))
stage_fused_kernel(const FusedItem* __restrict__ items, QuantDesc q1, StageDesc s1)
{
    extern __shared__ int lds[];
    constexpr int W = kFusedWaves;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, n = lane & 15;
    int rb = blockIdx.x;
    QuantDesc qd = q1;
    StageDesc sd = s1;
    if (LIST) {
        const FusedItem* e = items + blockIdx.x;           // uniform address of a kernel argument: scalar loads
        rb = e->rb;
        qd = e->q;
        sd = e->s;
    }
    const int nst = sd.n_steps;
    char* const lds_bq = (char*)lds;
    const size_t main_bytes = fused_lds_bytes(nst) - kFusedScratchInts * 4;
    float* const red_f = (float*)((char*)lds + main_bytes);                 // [W] partial maxima
    int* const red_bad = (int*)(red_f + W);                                 // the token holds a non-finite value
    double* const red_d = (double*)(red_f + W + 2);                         // [W] partial sums of q
    QMeta* const own_meta = (QMeta*)(red_d + W);                            // the token's constants
    static_assert((kFusedWaves + 2) * 4 + kFusedWaves * 8 + sizeof(QMeta) <= kFusedScratchInts * 4, "scratch region");

    // this wave's steps: wave, wave + W, ...; the first up to four tiles go out before anything else
    const int cnt = (nst - wave + W - 1) / W;
    const char* a_base = (const char*)sd.tiles + (size_t)rb * nst * (kTileWords * 4);
    v4u wbuf[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int st = cnt > 0 ? wave + (k < cnt ? k : cnt - 1) * W : 0;
        wbuf[k] = load_tile_words(a_base, (uint32_t)(st * 1024 + lane * 16));
    }

    // the output scales of this lane's two rows, needed last, are requested first
    // (an unconditional load, so that the compiler finds no branch to convert -- and wait -- inside:
    // a stage without output scales reads the start of its first tile instead and ignores it; the
    // scale array is padded to whole row blocks)
    uint16_t pre_scale[2];
    {
        const gptr_u16 sp = sd.out_scale ? (gptr_u16)sd.out_scale + rb * kTileRows : (gptr_u16)a_base;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) pre_scale[hf] = sp[64 * hf + lane];
    }

    // ---- quantise the input vector (as quantize_kernel does): thread tid owns chunk tid ----
    const int esz = qd.dtype == NQ_F32 ? 4 : 2;
    const bool vec = (((size_t)qd.x_stride * esz) & 15) == 0;
    const bool mine = tid < qd.n_chunks;
    float v[16];
    float m = 0.f;
    int bad = 0;
    if (tid == 0) *red_bad = 0;
    if (mine) {
        load_chunk16(qd, 0, tid, vec, v);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float a = fabsf(v[i]);
            if (!(a <= 3.0e38f)) bad = 1;
            m = fmaxf(m, a);
        }
    }
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (lane == 0) red_f[wave] = m;
    __syncthreads();
    if (bad) *red_bad = 1;
    __syncthreads();
    m = red_f[0];
#pragma unroll
    for (int w = 1; w < W; ++w) m = fmaxf(m, red_f[w]);
    bad = *red_bad;
    int e = 0;
    float step = 1.0f;
    if (m > 0.f && !bad) {
        (void)frexpf(m, &e);
        int se = e - 22;
        se = se < -126 ? -126 : se;
        step = ldexpf(1.0f, se);
    }
    const float inv_step = 1.0f / step;
    long long local_sum = 0;
    if (mine) local_sum = quantize_chunk16(v, inv_step, bad != 0, (uint4*)lds_bq + bq_piece(tid, 0));
    double sum = (double)local_sum;
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) red_d[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (int w = 0; w < W; ++w) tot += red_d[w];
        // the constants stay in the workgroup (LDS): its epilogue is their only reader
        own_meta->two_step = bad ? (double)__builtin_nanf("") : 2.0 * (double)step;
        own_meta->neg_qs = -tot * (double)step;
    }
    __syncthreads();
    const QMeta my_meta = *own_meta;

    // ---- the reduction over this wave's steps, operands from LDS ----
    const uint32_t b_lds = (uint32_t)(bq_piece(g, n < 3 ? n : 0) * 16);      // token 0; unused columns re-read slice 0
    v4i acc[1][8];
#pragma unroll
    for (int p = 0; p < 8; ++p) acc[0][p] = v4i{0, 0, 0, 0};
    for (int i0 = 0; i0 < cnt; i0 += 4) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i0 + k < cnt) {
                const int st = wave + (i0 + k) * W;
                v4u b[1];
                b[0] = *(const v4u*)(lds_bq + b_lds + st * (int)kBqStepBytes);
                mac_tile<1>(acc, wbuf[k], b);
                if (i0 + k + 4 < cnt) wbuf[k] = load_tile_words(a_base, (uint32_t)((st + 4 * W) * 1024 + lane * 16));
            }
        }
    }
    __syncthreads();                                       // the epilogue regions overlay the quantised input
    EpilogueArgs ea;
    ea.meta = sd.meta; ea.out_scale = sd.out_scale; ea.out = sd.out;
    ea.M = sd.M; ea.out_stride = sd.out_stride; ea.out_dtype = sd.out_dtype;
    stage_epilogue<1, W, false>(acc, lds, wave, lane, 1, rb, ea, nullptr, pre_scale, &my_meta);
}

#undef NQ_LOAD_ITEM

static int g_cu_count = 0;
int device_cu_count()
{
    if (g_cu_count == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            g_cu_count = prop.multiProcessorCount;
        if (g_cu_count <= 0) g_cu_count = 256;
    }
    return g_cu_count;
}

// tiles a wave of stage_selfq_kernel<W> keeps in flight (with the B operand in LDS a lone wave affords eight;
// measured on the 1024-layer pool: 192-193 us per step with 8 / 4, 194-195 us with 8 / 8, 6 / 6 or four waves per SIMD)
constexpr int kSelfqDepth1 = 8, kSelfqDepth4 = 4;
constexpr int kRingDepth = 4;        // the tile layout pads every reduction to a multiple of this many steps

template <int NB>
static int launch_stream_t(const StageDesc* d_descs, const StageDesc& single, const WorkItem* d_items, int n_items,
                           int rbs_per_item, int max_rbs_per_item, int batch, hipStream_t s)
{
    size_t lds_bytes = (size_t)kEpiRegion * sizeof(int) + (size_t)max_rbs_per_item * kTileRows * batch * sizeof(float);
    if (n_items < 1) return NQ_OK;
    NQ_LAUNCH((stage_stream_kernel<NB, kRingDepth>), dim3(n_items), dim3(64), lds_bytes, s, d_descs, single,
                       d_items, n_items, rbs_per_item, batch);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

template <int NB, int W>
static int launch_split_t(const StageDesc* d_descs, const StageDesc& single, const WorkItem* d_items, int n_items,
                          int batch, hipStream_t s)
{
    size_t lds_bytes = (size_t)W * kEpiRegion * sizeof(int);
    if (n_items < 1) return NQ_OK;
    NQ_LAUNCH((stage_split_kernel<NB, W, (NB == 1 ? kRingDepth : 2 * kRingDepth)>), dim3(n_items), dim3(64 * W), lds_bytes, s, d_descs,
                       single, d_items, n_items, batch);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// Row blocks per wave of the shared schedule: bounded by the LDS left for deferred results.
int shared_max_per(int batch)
{
    const int budget = batch > 5 ? kShareLdsBytes : (batch == 5 ? 52 : 39) * 1024;      // 2, 3 or 4 workgroups per CU
    const int left = budget - 2 * batch * kShareTokStride - kShareWaves * kEpiRegion * 4;
    const int per = left / (kShareWaves * kTileRows * 4 * batch);
    return std::max(1, std::min(per, 4));
}

// rows blocks per wave for an op with `nst` steps per row block (see stage_shared_kernel)
int shared_per_wave(int nst, int batch)
{
    if (nst % 8 != 0) return 1;                       // a half pass must be the last thing a wave does
    return std::max(1, std::min(shared_max_per(batch), stream_target_steps(batch) / std::max(1, nst)));
}

template <int NB, bool RESIDENT, int SL = 3>
static int launch_shared_t(const StageDesc* d_descs, const WorkItem* d_items, int n_items, int batch, hipStream_t s)
{
    static bool attr_set = false;
    const int per_max = shared_max_per(batch);
    const size_t lds_bytes = (size_t)2 * batch * kShareTokStride + (size_t)kShareWaves * kEpiRegion * 4 +
                             (size_t)kShareWaves * per_max * kTileRows * batch * 4;
    if (!d_items) {
        set_error("launch_stage: the shared schedule needs a work list");
        return NQ_E_INVALID_ARG;
    }
    if (n_items < 1) return NQ_OK;
    if (!attr_set) {
        NQ_HIP(hipFuncSetAttribute((const void*)stage_shared_kernel<NB, RESIDENT, SL>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   160 * 1024));
        attr_set = true;
    }
    NQ_LAUNCH((stage_shared_kernel<NB, RESIDENT, SL>), dim3(n_items), dim3(64 * kShareWaves), lds_bytes, s, d_descs, d_items,
                       n_items, per_max, batch);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// One stage of a lone layer at batch 1 together with the quantisation of its input (stage_fused_kernel).
bool fused_fits(int nst, int batch) { return batch == 1 && nst * 4 <= 64 * kFusedWaves; }

static int fused_set_attr()
{
    static bool attr_set = false;
    if (!attr_set) {
        NQ_HIP(hipFuncSetAttribute((const void*)stage_fused_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
        NQ_HIP(hipFuncSetAttribute((const void*)stage_fused_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
        attr_set = true;
    }
    return NQ_OK;
}

int launch_fused(const QuantDesc& q, const StageDesc& sd, hipStream_t s)
{
    int rc = fused_set_attr();
    if (rc != NQ_OK) return rc;
    hipLaunchKernelGGL(stage_fused_kernel<false>, dim3((unsigned)n_rowblocks(sd.M)), dim3(64 * kFusedWaves),
                       fused_lds_bytes(sd.n_steps), s, nullptr, q, sd);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// The same for a list of ops: one workgroup per item; `max_steps` is the longest reduction among
// the ops (it sizes the LDS of every workgroup).
int launch_fused_list(const FusedItem* d_items, int n_items, int max_steps, hipStream_t s)
{
    if (n_items < 1) return NQ_OK;
    if (!fused_fits(max_steps, 1)) {
        set_error("launch_fused_list: reduction too long for the fused kernel");
        return NQ_E_INVALID_ARG;
    }
    int rc = fused_set_attr();
    if (rc != NQ_OK) return rc;
    NQ_LAUNCH(stage_fused_kernel<true>, dim3((unsigned)n_items), dim3(64 * kFusedWaves),
                       fused_lds_bytes(max_steps), s, d_items, QuantDesc{}, StageDesc{});
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// Whether a batch-1 launch with schedule w (1 or 4) may quantise in the stage kernel: a wave's share
// of every reduction must be at most 16 steps (see stage_selfq_kernel; 32 with one wave per row block,
// whose lanes then hold two chunks), and with one wave per row block the reductions must not be so
// short that the stream kernel would chain row blocks.
bool selfq_fits(int w, int max_steps, int min_steps, int batch)
{
    if (batch != 1 || (w != 1 && w != 4)) return false;
    if (w == 1) return min_steps >= 16 && max_steps <= (opt_flag(OPT_NO_SELFQ_C2) ? 16 : 32);    // (two chunks per lane beyond 16)
    return max_steps <= 16 * w;
}

// Waves per row block (1 or 4) with which a batch-1 launch that does NOT fill the chip quantises in
// the stage kernel, 0 if its reductions are too long for that.  Such a launch is bound by the
// latency of its dependent launches and of a wave's chain of steps, so every length that fits is
// taken (short ones too), with four waves unless every reduction is exactly one wave's 16 steps.
int selfq_width(int max_steps, int min_steps, int batch)
{
    if (batch != 1) return 0;
    if (max_steps <= 16 && min_steps >= 16) return 1;
    return max_steps <= 64 ? 4 : 0;
}

// d_items == nullptr: the n_items row blocks of the one op (q1, s1).
int launch_selfq(const FusedItem* d_items, int n_items, const QuantDesc& q1, const StageDesc& s1, int w, int max_steps,
                 hipStream_t s)
{
    if (n_items < 1) return NQ_OK;
    if (!selfq_fits(w, max_steps, 16, 1)) {
        set_error("launch_selfq: schedule or reduction length not supported");
        return NQ_E_INVALID_ARG;
    }
    const int c = (w == 1 && max_steps > 16) ? 2 : 1;       // chunks a lane holds
    const size_t lds_bytes = (size_t)w * selfq_region_ints(c) * 4 + (w > 1 ? 2 * w * 4 : 0);     // + the waves' maxima and flags
    const dim3 grid((unsigned)n_items);
    if (w == 1 && c == 2 && d_items)
        NQ_LAUNCH((stage_selfq_kernel<1, kSelfqDepth1, true, 2>), grid, dim3(64), lds_bytes, s, d_items, q1, s1);
    else if (w == 1 && c == 2)
        NQ_LAUNCH((stage_selfq_kernel<1, kSelfqDepth1, false, 2>), grid, dim3(64), lds_bytes, s, d_items, q1, s1);
    else if (w == 1 && d_items)
        NQ_LAUNCH((stage_selfq_kernel<1, kSelfqDepth1, true>), grid, dim3(64), lds_bytes, s, d_items, q1, s1);
    else if (w == 1)
        NQ_LAUNCH((stage_selfq_kernel<1, kSelfqDepth1, false>), grid, dim3(64), lds_bytes, s, d_items, q1, s1);
    else if (d_items)
        NQ_LAUNCH((stage_selfq_kernel<4, kSelfqDepth4, true>), grid, dim3(256), lds_bytes, s, d_items, q1, s1);
    else
        NQ_LAUNCH((stage_selfq_kernel<4, kSelfqDepth4, false>), grid, dim3(256), lds_bytes, s, d_items, q1, s1);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// Row blocks from which a launch counts as filling the chip.
int schedule_full_rowblocks()
{
    const int v = opt(OPT_SCHEDULE_FULL);
    return v > 0 ? v : device_cu_count() * 8;
}

// Smallest batch whose long reductions take the shared-input kernel in launches that fill the chip.
// With one column group (batch <= 5) it pays from batch 4 on (stage 1 of the 4096x4096 r=1024 pool:
// 121 -> 116 us at batch 4, 130 -> 120 us at batch 5; batch 3 the same, batch 2 slower); short
// reductions (the resident variant) stay with the stream kernel below batch 6 (115 against 119 us).
int shared_min_batch() { return std::max(1, opt_or(OPT_SHARE_MIN_BATCH, 4)); }

int stage_schedule(int n_rb_total, int mean_steps, int batch)
{
    // row blocks from which a launch counts as filling the chip (NQ_SCHEDULE_FULL overrides it,
    // which lets small inputs exercise the schedules built for large launches)
    const int full = schedule_full_rowblocks();
    int w;
    if (n_rb_total >= full && batch >= shared_min_batch()) w = mean_steps >= std::max(1, opt_or(OPT_SHARE_STEPS, 32)) ? kSharedSchedule : 1;
    // (batch 1 splits from 33 steps on: stage 2 of the 70B stack, 35 and 55 steps, 452 -> 442 us; pools
    // of 35- and 55-step reductions 64 -> 62 and 91 -> 85 us including the quantisation launch)
    else if (n_rb_total >= full) w = mean_steps >= std::max(1, opt_or(OPT_SPLIT_STEPS, batch == 1 ? 33 : 64)) ? 4 : 1;
    else w = (n_rb_total * 4 >= full || batch > 2) ? 4 : 16;
    {
        const int fw = opt(OPT_FORCE_W);
        if (fw == 1 || fw == 4 || (fw == 16 && batch <= 2)) w = fw;     // (the shared schedule cannot be forced: it needs a work list)
    }
    return w;
}

// Steps one wave of the stream kernel should see per item (row blocks shorter than this are chained).
// Measured: beyond very short reductions chaining loses; many short items, whose epilogues and
// stores overlap with the streaming of the other waves, beat few long ones (stage 2 of the
// 4096x4096 r=1024 pool: 99.7 us with one 16-step row block per item, 103.5 us with eight).
// With two column groups (batch 6..8, two waves per SIMD) a few chained row blocks still pay (stage 2 of the
// same pool at batch 8: 197 us with three per item, 205 us with one).
int stream_target_steps(int batch) { return std::max(1, opt_or(OPT_STREAM_STEPS, batch <= 5 ? 16 : 64)); }

// Row blocks an item may chain: its deferred results (128 x batch floats per row block) share the
// CU's LDS with those of the other resident waves (20 per CU with one column group, 8 with two).
int stream_max_rbs(int batch)
{
    const int per = batch <= 5 ? kStreamMaxRbs / batch : 30 / batch;
    return std::max(1, std::min(per, kStreamMaxRbs));
}

int launch_stage(const StageDesc* d_descs, const StageDesc& single, const WorkItem* d_items, int n_items,
                 int w, int rbs_per_item, int batch, hipStream_t s)
{
    const int nb = batch <= 5 ? 1 : 2;
    if (w == kSharedSchedule2 || w == kSharedResidentSchedule2) {
        if (batch < 6 || batch > 8) {
            set_error("launch_stage: the two-slice schedules are for batch 6..8");
            return NQ_E_INVALID_ARG;
        }
        if (w == kSharedSchedule2) return launch_shared_t<1, false, 2>(d_descs, d_items, n_items, batch, s);
        return launch_shared_t<1, true, 2>(d_descs, d_items, n_items, batch, s);
    }
    if (w == kSharedSchedule || w == kSharedResidentSchedule) {
        if (nb == 1) {
            if (w == kSharedSchedule) return launch_shared_t<1, false>(d_descs, d_items, n_items, batch, s);
            return launch_shared_t<1, true>(d_descs, d_items, n_items, batch, s);
        }
        if (w == kSharedSchedule) return launch_shared_t<2, false>(d_descs, d_items, n_items, batch, s);
        return launch_shared_t<2, true>(d_descs, d_items, n_items, batch, s);
    }
    if (w == 1) {
        const int mx = stream_max_rbs(batch);
        if (rbs_per_item > mx) {
            set_error("launch_stage: item longer than the stream kernel's output buffer");
            return NQ_E_INVALID_ARG;
        }
        if (nb == 1) return launch_stream_t<1>(d_descs, single, d_items, n_items, rbs_per_item, mx, batch, s);
        return launch_stream_t<2>(d_descs, single, d_items, n_items, rbs_per_item, mx, batch, s);
    }
    if (nb == 1) {
        if (w == 4) return launch_split_t<1, 4>(d_descs, single, d_items, n_items, batch, s);
        return launch_split_t<1, 16>(d_descs, single, d_items, n_items, batch, s);
    }
    return launch_split_t<2, 4>(d_descs, single, d_items, n_items, batch, s);
}

// ---------------------------------------------------------------------------------------------
// out[j] = sum_b a[b][j] * b[b][j]: the reduction over the batch that turns an upstream gradient
// and an unscaled product into the gradient of a scale vector (Section 3.4: the scales are tuned
// with the packed signs frozen).  One thread per column, fp64 accumulation, one rounding.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
scale_grad_kernel(const void* __restrict__ a, int a_dtype, const void* __restrict__ b, int b_dtype, int batch, int64_t n,
                  float* __restrict__ out)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    double acc = 0.0;
    for (int t = 0; t < batch; ++t)
        acc += (double)load_as_float(a, a_dtype, (int64_t)t * n + j) * (double)load_as_float(b, b_dtype, (int64_t)t * n + j);
    out[j] = (float)acc;
}

int launch_scale_grad(const void* a, int a_dtype, const void* b, int b_dtype, int batch, int64_t n, float* out, hipStream_t s)
{
    hipLaunchKernelGGL(scale_grad_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a, a_dtype, b, b_dtype, batch, n, out);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// ---------------------------------------------------------------------------------------------
// plain vector-ALU GEMV on the same sign tiles: one thread per output row, fp32 accumulate,
// bit -> sign by mask and select, then a multiply-add: the plain vector-ALU form of the two-stage product that Appendix E.2 describes.
// grid = (row blocks, batch), block = 128
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(128)
valu_gemv_kernel(const uint32_t* __restrict__ tiles, const void* __restrict__ x, int x_dtype, int x_stride,
                 const uint16_t* __restrict__ in_scale, const uint16_t* __restrict__ out_scale,
                 void* __restrict__ out, int out_dtype, int out_stride, int64_t M, int64_t N, int64_t nsteps)
{
    const int rr = threadIdx.x;                     // row inside the block
    const int64_t rb = blockIdx.x, tok = blockIdx.y;
    const int p = rr >> 4, i16 = rr & 15;
    const int64_t row = rb * kTileRows + rr;
    float acc = 0.f;
    for (int64_t st = 0; st < nsteps; ++st) {
        const uint32_t* tile = tiles + ((size_t)rb * nsteps + st) * kTileWords;
        for (int g = 0; g < 4; ++g)
            for (int v = 0; v < 4; ++v) {
                uint32_t w = tile[(g * 16 + i16) * 4 + v];
                for (int b = 0; b < 4; ++b) {
                    int64_t col = st * kTileCols + 16 * g + 4 * v + b;
                    if (col < N) {
                        float xv = load_as_float(x, x_dtype, tok * x_stride + col);
                        if (in_scale) xv *= half_bits_to_float(in_scale[col]);
                        acc += ((w >> (8 * b + p)) & 1u) ? xv : -xv;
                    }
                }
            }
    }
    if (row < M) {
        if (out_scale) acc *= half_bits_to_float(out_scale[row]);
        store_out(out, out_dtype, (size_t)tok * out_stride + row, acc);
    }
}

int launch_valu_gemv(const uint32_t* tiles, const void* x, int x_dtype, int x_stride, const uint16_t* in_scale,
                     const uint16_t* out_scale, void* out, int out_dtype, int out_stride, int64_t M, int64_t N, int batch,
                     hipStream_t s)
{
    hipLaunchKernelGGL(valu_gemv_kernel, dim3((unsigned)n_rowblocks(M), batch), dim3(128), 0, s, tiles, x, x_dtype,
                       x_stride, in_scale, out_scale, out, out_dtype, out_stride, M, N, n_steps(N));
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

}  // namespace nq
