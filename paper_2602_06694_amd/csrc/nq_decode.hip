// Streaming (decode, batch <= 8) kernels of the two-stage binary product
//     t = V^T (s_in (.) x),   y = s_out (.) (U t)          (Section 3.1 Eq. 1; Appendix D, GEMV)
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
#include "nq_internal.h"

namespace nq {

typedef int v4i __attribute__((ext_vector_type(4)));

__device__ inline float half_bits_to_float(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ inline float bf16_bits_to_float(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }

__device__ inline float load_as_float(const void* p, int dtype, int64_t idx)
{
    if (dtype == NQ_F32) return ((const float*)p)[idx];
    if (dtype == NQ_F16) return half_bits_to_float(((const uint16_t*)p)[idx]);
    return bf16_bits_to_float(((const uint16_t*)p)[idx]);
}

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
// grid = (n_ops, batch), block = 256
// ---------------------------------------------------------------------------------------------
__device__ inline float block_max(float v, float* sm)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    __syncthreads();
    return r;
}

__global__ void __launch_bounds__(256)
quantize_kernel(const QuantDesc* __restrict__ descs, QuantDesc single, int batch)
{
    __shared__ float smf[4];
    __shared__ double smd[4];
    const QuantDesc d = descs ? descs[blockIdx.x] : single;
    const int tok = blockIdx.y;
    const int ncols = ncols_for(batch);
    const int64_t base = (int64_t)tok * d.x_stride;

    // pass 1: max |v|; any NaN/Inf is remembered separately (fmaxf drops NaN)
    float m = 0.f;
    int bad = 0;
    for (int j = threadIdx.x; j < d.N; j += 256) {
        float v = load_as_float(d.x, d.dtype, base + j);
        if (d.scale) v *= half_bits_to_float(d.scale[j]);
        if (!(fabsf(v) <= 3.0e38f)) bad = 1;
        m = fmaxf(m, fabsf(v));
    }
    m = block_max(m, smf);
    bad = __syncthreads_or(bad);

    // step = 2^(e-22) with m = f * 2^e, f in [0.5, 1)  ->  |q| <= 2^22
    int e = 0;
    float step = 1.0f;
    if (m > 0.f) {
        (void)frexpf(m, &e);
        int se = e - 22;
        se = se < -126 ? -126 : se;            // stay a normal float; tiny inputs just lose bits
        step = ldexpf(1.0f, se);
    }
    const float inv_step = 1.0f / step;        // exact: power of two

    // pass 2: q = rint(v / step), split into three signed bytes, write the MFMA B-operand layout
    long long local_sum = 0;
    const int c0 = col_of(tok, 0);
    for (int c = threadIdx.x; c < d.n_chunks; c += 256) {
        uint32_t hi[4] = {0, 0, 0, 0}, mid[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
        for (int i = 0; i < 16; ++i) {
            int j = c * 16 + i;
            int q = 0;
            if (j < d.N && !bad) {
                float v = load_as_float(d.x, d.dtype, base + j);
                if (d.scale) v *= half_bits_to_float(d.scale[j]);
                q = (int)rintf(v * inv_step);
            }
            local_sum += q;
            int l = ((q + 128) & 255) - 128;
            int q1 = (q - l) >> 8;
            int mm = ((q1 + 128) & 255) - 128;
            int h = (q1 - mm) >> 8;
            int sh = 8 * (i & 3);
            hi[i >> 2] |= (uint32_t)(h & 255) << sh;
            mid[i >> 2] |= (uint32_t)(mm & 255) << sh;
            lo[i >> 2] |= (uint32_t)(l & 255) << sh;
        }
        uint4* dst = (uint4*)(d.bq) + ((size_t)c * ncols + c0);
        dst[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        dst[1] = make_uint4(mid[0], mid[1], mid[2], mid[3]);
        dst[2] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
    double s = (double)local_sum;               // |sum| < 2^39: exact
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if ((threadIdx.x & 63) == 0) smd[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        QMeta mt;
        mt.sumq = smd[0] + smd[1] + smd[2] + smd[3];
        mt.step = bad ? __builtin_nanf("") : step;
        mt.pad = 0.f;
        d.meta[tok] = mt;
    }
}

int launch_quantize(const QuantDesc* d_descs, const QuantDesc& single, int n_ops, int batch, hipStream_t s)
{
    hipLaunchKernelGGL(quantize_kernel, dim3(n_ops, batch), dim3(256), 0, s, d_descs, single, batch);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// ---------------------------------------------------------------------------------------------
// streaming sign-matrix x fixed-point-vector kernel (steps a2 and a4, with a5 fused in stage 2)
//   NB : number of 16-column groups of the B operand (1: batch <= 5, 2: batch 6..8)
//   W  : wavefronts that share one work item (1: every wave walks its own items;
//        4 / 16: the workgroup's waves interleave the 64-column steps of one item and are
//        summed through LDS -- for launches with too few items to fill the chip)
//   D  : software prefetch depth (tiles in flight per wave)
// A work item is one 128-row block of one op, over the whole reduction length.
// ---------------------------------------------------------------------------------------------
#ifndef NQ_STAGE_WAVES
#define NQ_STAGE_WAVES 4
#endif
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// streamed once, never reused: keep the sign tiles from displacing the (reused) activations in cache
typedef const __attribute__((address_space(1))) v4u* gptr_v4u;    // global (not generic) address space
__device__ inline v4u load_tile_words(const char* base, uint32_t off)
{
    return __builtin_nontemporal_load((gptr_v4u)(base + off));
}
__device__ inline v4u load_global_v4u(const char* base, uint32_t off) { return *(gptr_v4u)(base + off); }

template <int NB, int W, int D>
__global__ void __launch_bounds__(W == 1 ? 256 : 64 * W) __attribute__((amdgpu_waves_per_eu(NB == 1 ? NQ_STAGE_WAVES : 2, 8)))
stage_kernel(const StageDesc* __restrict__ descs, StageDesc single, const WorkItem* __restrict__ items, int n_items,
             int batch)
{
    extern __shared__ int lds[];
    constexpr int WPB = (W == 1) ? 4 : W;               // waves per block
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int ncols = ncols_for(batch);
    int* my_lds = lds + wave * (kTileRows * ncols);

    const int stream = (W == 1) ? (int)blockIdx.x * WPB + wave : (int)blockIdx.x;
    const int nstreams = (W == 1) ? (int)gridDim.x * WPB : (int)gridDim.x;
    const int st0 = (W == 1) ? 0 : wave;

    for (int it = stream; it < n_items; it += nstreams) {
        // descriptor fields are wave-uniform: fetch them with scalar loads
        const uint32_t* tiles;
        const uint8_t* bq;
        const QMeta* meta;
        const uint16_t* out_scale;
        float* out;
        int M, nst, out_stride, rb;
        if (items) {
            const WorkItem e = items[it];
            const StageDesc* dp = descs + e.op;
            rb = e.rb;
            tiles = dp->tiles; bq = dp->bq; meta = dp->meta; out_scale = dp->out_scale; out = dp->out;
            M = dp->M; nst = dp->n_steps; out_stride = dp->out_stride;
        } else {
            rb = it;
            tiles = single.tiles; bq = single.bq; meta = single.meta; out_scale = single.out_scale; out = single.out;
            M = single.M; nst = single.n_steps; out_stride = single.out_stride;
        }
        const int cnt = (nst - st0 + W - 1) / W;         // steps this wave performs (may be <= 0)
        // 32-bit byte offsets from the (scalar) base pointers; a tile array is at most 512 MiB
        // (a wave with no step of its own, possible when W > nst, aims its unused prefetches at step 0)
        const int stf = cnt > 0 ? st0 : 0;
        uint32_t a_off = (uint32_t)(((size_t)rb * nst + stf) * 1024 + lane * 16);
        // lanes whose column is beyond ncols re-read column 0: their result columns are never used
        uint32_t b_off[NB];
#pragma unroll
        for (int cg = 0; cg < NB; ++cg) {
            int col = cg * 16 + n;
            b_off[cg] = (uint32_t)(((stf * 4 + g) * ncols + (col < ncols ? col : 0)) * 16);
        }
        const uint32_t b_inc = (uint32_t)(W * 4 * ncols * 16);
        const char* a_base = (const char*)tiles;
        const char* b_base = (const char*)bq;

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
#define NQ_COMPUTE(w, b)                                                         \
    do {                                                                         \
        _Pragma("unroll") for (int p = 0; p < 8; ++p) {                          \
            const uint32_t mask = 0x01010101u << p;                              \
            const v4i a = (v4i)((w) & mask);                                     \
            _Pragma("unroll") for (int cg = 0; cg < NB; ++cg)                    \
                acc[cg][p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, (v4i)(b)[cg], acc[cg][p], 0, 0, 0); \
        }                                                                        \
    } while (0)

        // prologue: D tiles in flight.  Issued unconditionally and branch-free (a short item
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
                NQ_COMPUTE(wbuf[k], bbuf[k]);
                NQ_ISSUE(k);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // last D..2D-1 steps: refill only while tiles remain
#pragma unroll
        for (int k = 0; k < D; ++k) {
            if (i0 + k < cnt) {
                NQ_COMPUTE(wbuf[k], bbuf[k]);
                if (i0 + k + D < cnt) NQ_ISSUE(k);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int k = 0; k < D; ++k) {
            if (i0 + D + k < cnt) {
                NQ_COMPUTE(wbuf[k], bbuf[k]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#undef NQ_ISSUE
#undef NQ_COMPUTE

        // ---- epilogue: raw accumulators -> LDS [row][col], then one thread per (token, row) ----
        // accumulator layout of the 16x16 result: lane (g, n), register v  <->  D[row 4g+v][col n]
#pragma unroll
        for (int cg = 0; cg < NB; ++cg) {
            int col = cg * 16 + n;
            if (col < ncols) {
#pragma unroll
                for (int p = 0; p < 8; ++p)
#pragma unroll
                    for (int v = 0; v < 4; ++v) my_lds[(16 * p + 4 * g + v) * ncols + col] = acc[cg][p][v];
            }
        }
        if (W == 1) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        } else {
            __syncthreads();
        }
        constexpr int T = (W == 1) ? 64 : 64 * W;          // threads that cooperate on the outputs
        const int tid = (W == 1) ? lane : (int)threadIdx.x;
        const int* src = (W == 1) ? my_lds : lds;
        for (int o = tid; o < kTileRows * batch; o += T) {
            int row = o & (kTileRows - 1), tok = o >> 7;
            int c0 = col_of(tok, 0);
            int h = 0, m = 0, l = 0;
#pragma unroll
            for (int w = 0; w < (W == 1 ? 1 : W); ++w) {
                const int* q = src + w * (kTileRows * ncols) + row * ncols + c0;
                h += q[0];
                m += q[1];
                l += q[2];
            }
            // plane p holds 2^p * sum (p < 7) or -128 * sum (p = 7, the int8 sign bit): exact shifts
            int p = row >> 4;
            h >>= p;
            m >>= p;
            l >>= p;
            if (p == 7) {
                h = -h;
                m = -m;
                l = -l;
            }
            double bsum = fma((double)h, 65536.0, fma((double)m, 256.0, (double)l));   // sum_n b_n q_n
            QMeta mt = meta[tok];
            double val = (2.0 * bsum - mt.sumq) * (double)mt.step;
            int grow = rb * kTileRows + row;
            if (grow < M) {
                if (out_scale) val *= (double)half_bits_to_float(out_scale[grow]);
                out[(size_t)tok * out_stride + grow] = (float)val;
            }
        }
        if (W == 1) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
        } else {
            __syncthreads();
        }
    }
}

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

static int env_int(const char* name, int dflt)
{
    const char* v = getenv(name);
    if (!v || !*v) return dflt;
    int x = atoi(v);
    return x > 0 ? x : dflt;
}

template <int NB, int W>
static int launch_stage_t(const StageDesc* d_descs, const StageDesc& single, const WorkItem* d_items, int n_items,
                          int batch, hipStream_t s)
{
    constexpr int D = (NB == 1) ? 4 : 4;
    constexpr int WPB = (W == 1) ? 4 : W;
    const int ncols = ncols_for(batch);
    size_t lds_bytes = (size_t)WPB * kTileRows * ncols * sizeof(int);
    int blocks;
    if (W == 1) {
        int per_cu = env_int("NQ_WG_PER_CU", 4);
        int cap = device_cu_count() * per_cu;
        blocks = (n_items + WPB - 1) / WPB;
        if (blocks > cap) blocks = cap;
    } else {
        blocks = n_items;
    }
    if (blocks < 1) return NQ_OK;
    hipLaunchKernelGGL((stage_kernel<NB, W, D>), dim3(blocks), dim3(64 * WPB), lds_bytes, s, d_descs, single, d_items,
                       n_items, batch);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

int launch_stage(const StageDesc* d_descs, const StageDesc& single, const WorkItem* d_items, int n_items, int batch,
                 hipStream_t s)
{
    const int nb = batch <= 5 ? 1 : 2;
    // enough independent items to give every SIMD of the chip a few waves?  then one wave per item
    const int full = device_cu_count() * 8;
    int w = 1;
    if (n_items < full) w = (n_items * 4 >= full || batch > 2) ? 4 : 16;
    if (const char* f = getenv("NQ_FORCE_W")) {
        int fw = atoi(f);
        if (fw == 1 || fw == 4 || (fw == 16 && batch <= 2)) w = fw;
    }
    if (nb == 1) {
        if (w == 1) return launch_stage_t<1, 1>(d_descs, single, d_items, n_items, batch, s);
        if (w == 4) return launch_stage_t<1, 4>(d_descs, single, d_items, n_items, batch, s);
        return launch_stage_t<1, 16>(d_descs, single, d_items, n_items, batch, s);
    }
    if (w == 1) return launch_stage_t<2, 1>(d_descs, single, d_items, n_items, batch, s);
    return launch_stage_t<2, 4>(d_descs, single, d_items, n_items, batch, s);
}

// ---------------------------------------------------------------------------------------------
// plain vector-ALU GEMV on the same sign tiles: one thread per output row, fp32 accumulate,
// bit -> sign by mask and select (the paper-style "lightweight mask + FMA" kernel).
// grid = (row blocks, batch), block = 128
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(128)
valu_gemv_kernel(const uint32_t* __restrict__ tiles, const void* __restrict__ x, int x_dtype, int x_stride,
                 const uint16_t* __restrict__ in_scale, const uint16_t* __restrict__ out_scale,
                 float* __restrict__ out, int out_stride, int64_t M, int64_t N, int64_t nsteps)
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
        out[(size_t)tok * out_stride + row] = acc;
    }
}

int launch_valu_gemv(const uint32_t* tiles, const void* x, int x_dtype, int x_stride, const uint16_t* in_scale,
                     const uint16_t* out_scale, float* out, int out_stride, int64_t M, int64_t N, int batch,
                     hipStream_t s)
{
    hipLaunchKernelGGL(valu_gemv_kernel, dim3((unsigned)n_rowblocks(M), batch), dim3(128), 0, s, tiles, x, x_dtype,
                       x_stride, in_scale, out_scale, out, out_stride, M, N, n_steps(N));
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

}  // namespace nq
