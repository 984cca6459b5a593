// Dense (prefill, batch >= 9) path of  y = s_out (.) (U (V^T (s_in (.) x)))   (Section 3.1 Eq. 1;
// Appendix E.3, "Binary GEMM Inference"): both contractions run on the fp16 matrix cores of gfx950.
//
//   pre   : x'' = fp16( s_in (.) x * 2^a_b )          per token b, 2^a_b puts max|x''| in [2^12, 2^13)
//   gemm1 : T   = fp16( (X'' V) * g )                 g = power of two so that |T| <= 2^15 always
//   gemm2 : y   = (T U^T) (.) s_out / (2^a_b * g)     fp32 out
//
// The sign matrices stay in the 1-bit tile layout of the streaming kernels.  A wave owns 128
// output rows (one tile row block) and turns each 16-byte tile fragment in registers into the A
// operands of v_mfma_f32_16x16x32_f16 with ONE vector AND per two weights: a weight's bit is left
// where it is inside its 16-bit half, and a half with only bit p set IS an fp16 number, the
// denormal 2^(p-24), which the matrix cores take at full precision.  Plane p (rows 16p .. 16p+15)
// therefore accumulates 2^(p-24) * P with P = sum over the +1 weights of the activations, and the
// signed sum follows as 2P - S, S = the plain sum of the activations of the token (two-operand
// dot products on the chunks a thread stages anyway).  Against building +-1.0 operands (a shift
// and a bit-field insert per two weights) this halves the vector instructions beside the MFMAs;
// the two share the issue port of a SIMD, which was saturated.  The 64-token activation tile is
// shared by the four waves of a workgroup through LDS, and two workgroups share a CU (two waves
// per SIMD keep the matrix pipe fed).
//
// fp16 (not bf16) operands: +-1 is exact in both and the MFMA rate is the same, but rounding x'
// and t to 8 mantissa bits breaks the 1e-3 parity bar while 11 bits hold it with margin.
//
// Activation element order.  The two half2 registers made from one tile word hold reduction
// indices (k0, k2) and (k1, k3); instead of permuting registers, X'' and T are STORED with the
// middle two elements of every aligned group of four swapped, so a plain 16-byte LDS read yields
// the matching B operand.
#include <algorithm>
#include <cstdio>
#include <type_traits>

#include "nq_internal.h"

namespace nq {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u32 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) v4u32* gp_v4u32;

constexpr int kPfTokens = 64;           // tokens per workgroup tile (4 MFMA column groups)
constexpr int kPfWaves = 4;             // waves per workgroup, one 128-row block each
constexpr int kPfLdsStride = 72;        // halves per token row in LDS (64 + 8: conflict-free 16-byte reads)
constexpr int kPfThreads = 64 * kPfWaves;
constexpr int kPfTrStride = 132;        // floats per token row of a wave's epilogue region (128 + 4: conflict-free both ways)

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
enum { EPI_PARTIAL = 0, EPI_T = 1, EPI_Y = 2 };

struct GemmArgs {
    const _Float16* act;       // [m_pad][lda] halves, element order swizzled (see above)
    const uint32_t* tiles;     // sign tiles of the weight: rows = outputs, columns = reduction
    float* partial;            // EPI_PARTIAL: [splits][m_pad][n_pad] raw accumulators
    _Float16* t_out;           // EPI_T: [m_pad][ldt]
    void* y_out;               // EPI_Y: [batch][n_real] elements of y_dtype
    int y_dtype;
    const float* tok_scale;    // EPI_Y: per token 1 / (2^a_b * g)
    const uint16_t* out_scale; // EPI_Y: fp16 [n_real]
    float t_scale;             // EPI_T: g
    const uint16_t* mid_scale; // EPI_T: rank-wise scale fp16 [n_pad] (zeros beyond n_real) or nullptr
    int lda, ldt;
    int n_real;                // real output rows
    int n_rb;                  // row blocks of the weight
    int nst;                   // 64-column steps of the reduction
    int m_tiles, n_tiles;      // workgroup grid
    int batch;                 // real tokens
    int splits, steps_per_split;
    int n_pad, m_pad;
};

__device__ __forceinline__ float h2f(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

// ---------------------------------------------------------------------------------------------
// pre-scale: one workgroup per token
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float pf_load(const void* p, int dtype, int64_t i)
{
    if (dtype == NQ_F32) return ((const float*)p)[i];
    if (dtype == NQ_F16) return h2f(((const uint16_t*)p)[i]);
    return __builtin_bit_cast(float, (uint32_t)((const uint16_t*)p)[i] << 16);
}

// eight consecutive scaled inputs x'[k0..k0+7] of one token (zero beyond d_in)
__device__ __forceinline__ void pf_load8(const void* x, int dtype, const uint16_t* s_in, int64_t base, int k0, int d_in,
                                         bool vec, float v[8])
{
    if (vec && k0 + 8 <= d_in) {
        if (dtype == NQ_F32) {
            const float4 f0 = *(const float4*)((const float*)x + base + k0);
            const float4 f1 = *(const float4*)((const float*)x + base + k0 + 4);
            v[0] = f0.x; v[1] = f0.y; v[2] = f0.z; v[3] = f0.w; v[4] = f1.x; v[5] = f1.y; v[6] = f1.z; v[7] = f1.w;
        } else {
            const uint4 u = *(const uint4*)((const uint16_t*)x + base + k0);
            const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint16_t lo = (uint16_t)(w[i] & 0xFFFFu), hi = (uint16_t)(w[i] >> 16);
                v[2 * i] = dtype == NQ_F16 ? h2f(lo) : __builtin_bit_cast(float, (uint32_t)lo << 16);
                v[2 * i + 1] = dtype == NQ_F16 ? h2f(hi) : __builtin_bit_cast(float, (uint32_t)hi << 16);
            }
        }
        const uint4 su = *(const uint4*)(s_in + k0);
        const uint32_t sw[4] = {su.x, su.y, su.z, su.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] *= h2f((uint16_t)(sw[i] & 0xFFFFu));
            v[2 * i + 1] *= h2f((uint16_t)(sw[i] >> 16));
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = k0 + i < d_in ? pf_load(x, dtype, base + k0 + i) * h2f(s_in[k0 + i]) : 0.f;
    }
}

// one workgroup per token: max |x'|, then x'' = fp16(x' * 2^a) in the swizzled element order.
// Up to kPreHeld groups of eight values per thread stay in registers between the two passes
// (rows up to 32768 elements are read once); longer rows are read twice.
constexpr int kPreThreads = 1024;
constexpr int kPreHeld = 4;

__device__ __forceinline__ void pf_store8(_Float16* dst, const float v[8], float sc)
{
    // storage order inside every aligned group of four: 0, 2, 1, 3
    v8h o;
    o[0] = (_Float16)(v[0] * sc); o[1] = (_Float16)(v[2] * sc); o[2] = (_Float16)(v[1] * sc); o[3] = (_Float16)(v[3] * sc);
    o[4] = (_Float16)(v[4] * sc); o[5] = (_Float16)(v[6] * sc); o[6] = (_Float16)(v[5] * sc); o[7] = (_Float16)(v[7] * sc);
    *(v8h*)dst = o;
}

// DT: the element type of x (a template parameter, so that the loads of the fast path sit in
// straight-line code: all of a thread's chunks are requested back to back, then converted).
template <int DT>
__global__ void __launch_bounds__(kPreThreads)
prefill_prescale_kernel(const void* __restrict__ x, const uint16_t* __restrict__ s_in, int d_in, int lda,
                        float g_t, _Float16* __restrict__ xs, float* __restrict__ tok_scale)
{
    __shared__ float sm[kPreThreads / 64];
    constexpr int x_dtype = DT;
    const int tok = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)tok * d_in;
    constexpr int esz = DT == NQ_F32 ? 4 : 2;
    const bool vec = (((size_t)d_in * esz) & 15) == 0;      // every token row starts 16-byte aligned
    const int n8 = lda / 8;
    const bool held = n8 <= kPreThreads * kPreHeld;
    // rows of whole, aligned chunks (every model shape): no branch around a load.  A thread's chunk
    // past the end of the row re-reads chunk 0 and counts as zeros.
    const bool fast = held && vec && (d_in & 7) == 0;
    float hv[kPreHeld][8];
    float m = 0.f;
    if (fast) {
        const int n_in = d_in / 8;
        typedef const __attribute__((address_space(1))) v4f* gp_v4f;
        v4u32 xr0[kPreHeld], sr[kPreHeld];
        v4f xf0[kPreHeld], xf1[kPreHeld];
        const char* const xrow = (const char*)x + (size_t)base * esz;
#pragma unroll
        for (int k = 0; k < kPreHeld; ++k) {
            const int c = tid + k * kPreThreads;
            const uint32_t cc = (uint32_t)(c < n_in ? c : 0);
            if (DT == NQ_F32) {
                xf0[k] = *(gp_v4f)(xrow + cc * 32u);
                xf1[k] = *(gp_v4f)(xrow + cc * 32u + 16u);
            } else {
                xr0[k] = *(gp_v4u32)(xrow + cc * 16u);
            }
            sr[k] = *(gp_v4u32)((const char*)s_in + cc * 16u);
        }
#pragma unroll
        for (int k = 0; k < kPreHeld; ++k) {
            const bool valid = tid + k * kPreThreads < n_in;
            float xv[8];
            if (DT == NQ_F32) {
                const v4f a = xf0[k], b = xf1[k];
                xv[0] = a.x; xv[1] = a.y; xv[2] = a.z; xv[3] = a.w;
                xv[4] = b.x; xv[5] = b.y; xv[6] = b.z; xv[7] = b.w;
            } else {
                const uint32_t w[4] = {xr0[k].x, xr0[k].y, xr0[k].z, xr0[k].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint16_t lo = (uint16_t)(w[i] & 0xFFFFu), hi = (uint16_t)(w[i] >> 16);
                    xv[2 * i] = DT == NQ_F16 ? h2f(lo) : __builtin_bit_cast(float, (uint32_t)lo << 16);
                    xv[2 * i + 1] = DT == NQ_F16 ? h2f(hi) : __builtin_bit_cast(float, (uint32_t)hi << 16);
                }
            }
            const uint32_t sw[4] = {sr[k].x, sr[k].y, sr[k].z, sr[k].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float v0 = xv[2 * i] * h2f((uint16_t)(sw[i] & 0xFFFFu));
                const float v1 = xv[2 * i + 1] * h2f((uint16_t)(sw[i] >> 16));
                hv[k][2 * i] = valid ? v0 : 0.f;
                hv[k][2 * i + 1] = valid ? v1 : 0.f;
                m = fmaxf(m, fmaxf(fabsf(hv[k][2 * i]), fabsf(hv[k][2 * i + 1])));
            }
        }
    } else if (held) {
#pragma unroll
        for (int k = 0; k < kPreHeld; ++k) {
            const int c = tid + k * kPreThreads;
            if (c < n8) {
                pf_load8(x, x_dtype, s_in, base, c * 8, d_in, vec, hv[k]);
#pragma unroll
                for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(hv[k][i]));
            }
        }
    } else {
        for (int c = tid; c < n8; c += kPreThreads) {
            float v[8];
            pf_load8(x, x_dtype, s_in, base, c * 8, d_in, vec, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(v[i]));
        }
    }
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if ((tid & 63) == 0) sm[tid >> 6] = m;
    __syncthreads();
    m = sm[0];
#pragma unroll
    for (int w = 1; w < kPreThreads / 64; ++w) m = fmaxf(m, sm[w]);
    // 2^a with max * 2^a in [2^12, 2^13); a NaN/Inf token keeps a = 0 and poisons only itself
    float sc = 1.0f;
    if (m > 0.f && m <= 3.0e38f) {
        int e;
        (void)frexpf(m, &e);
        int a = 13 - e;
        a = a > 100 ? 100 : (a < -100 ? -100 : a);
        sc = ldexpf(1.0f, a);
    }
    _Float16* row = xs + (size_t)tok * lda;
    if (held) {
#pragma unroll
        for (int k = 0; k < kPreHeld; ++k) {
            const int c = tid + k * kPreThreads;
            if (c < n8) pf_store8(row + c * 8, hv[k], sc);
        }
    } else {
        for (int c = tid; c < n8; c += kPreThreads) {
            float v[8];
            pf_load8(x, x_dtype, s_in, base, c * 8, d_in, vec, v);
            pf_store8(row + c * 8, v, sc);
        }
    }
    if (tid == 0) tok_scale[tok] = 1.0f / (sc * g_t);
}

// ---------------------------------------------------------------------------------------------
// GEMM:  C[token][n] = sum_k act[token][k] * sign(tiles[n][k])
// grid = (m_tiles * n_tiles, splits); block = 256 (4 waves x 128 output rows, 64 tokens)
// ---------------------------------------------------------------------------------------------
// acc + the sum of the eight fp16 values of a 16-byte chunk (each times `ones`): four v_dot2_f32_f16
__device__ __forceinline__ float pf_sum8(const uint4& c, half2v ones, float acc)
{
    // (the words are copied out first: a bit cast applied directly to an element of a vector
    // type may read the vector's first element instead)
    const uint32_t w0 = c.x, w1 = c.y, w2 = c.z, w3 = c.w;
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, w0), ones, acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, w1), ones, acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, w2), ones, acc, false);
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, w3), ones, acc, false);
}

// One lane's four results of gemm 1 (rows n0 .. n0 + 3 of token `tok`, raw accumulators of negated
// signs) -> fp16 T: times g, times the rank-wise scale of the three-scale variant where there is
// one (its own power of two is folded into g), rows beyond the real rank exact zeros (they are
// padding of the next reduction); stored in the swizzled order 0, 2, 1, 3.
__device__ __forceinline__ void store_t(const GemmArgs& a, int tok, int n0, const v4f c)
{
    float f[4] = {-a.t_scale, -a.t_scale, -a.t_scale, -a.t_scale};
    if (a.mid_scale) {
        const uint2 m = *(const uint2*)(a.mid_scale + n0);
        f[0] *= h2f((uint16_t)(m.x & 0xFFFFu));
        f[1] *= h2f((uint16_t)(m.x >> 16));
        f[2] *= h2f((uint16_t)(m.y & 0xFFFFu));
        f[3] *= h2f((uint16_t)(m.y >> 16));
    }
    v4h o;
    o.x = (_Float16)(n0 + 0 < a.n_real ? c.x * f[0] : 0.f);
    o.y = (_Float16)(n0 + 2 < a.n_real ? c.z * f[2] : 0.f);
    o.z = (_Float16)(n0 + 1 < a.n_real ? c.y * f[1] : 0.f);
    o.w = (_Float16)(n0 + 3 < a.n_real ? c.w * f[3] : 0.f);
    *(v4h*)(a.t_out + (size_t)tok * a.ldt + n0) = o;
}

// TG = token groups of 16 per workgroup tile: 4 (64 tokens) normally; 2 (32 tokens) for narrow
// outputs at small batches, where 64-token tiles are too few to cover the chip and splitting the
// reduction instead would cost partial sums and a finalize pass (the sign expansion is then shared
// by half as many MFMAs: lower efficiency per workgroup, but no extra passes).
// KS = 2: eight waves; waves 4..7 take the same rows and tokens as waves 0..3 but the second half of
// the workgroup's part of the reduction (with activation buffers of their own), and hand their
// accumulators to their partners through LDS before the epilogue.  For GEMMs whose tiles (times
// splits) number no more than the CUs: such a workgroup fills its CU by itself (two waves per
// SIMD), and the reduction is halved without partial sums in memory.
template <int EPI, int TG, int KS = 1>
__global__ void __launch_bounds__(kPfThreads * KS) __attribute__((amdgpu_waves_per_eu(2, TG == 4 ? 2 : 4)))
prefill_gemm_kernel(GemmArgs a)
{
    static_assert(TG == 2 || TG == 4, "32- or 64-token tiles");
    static_assert(KS == 1 || (KS == 2 && TG == 4), "the in-workgroup split is built for 64-token tiles");
    constexpr int kTok = 16 * TG;
    // four activation buffers (per half of the workgroup); after the reduction the same memory serves
    // the exchange of accumulators and the epilogue
    constexpr int kActBuf = kTok * kPfLdsStride;                            // halves per buffer
    constexpr int kLdsBytes = KS * 4 * kActBuf * 2 > kPfWaves * 16 * kPfTrStride * 4 ? KS * 4 * kActBuf * 2 : kPfWaves * 16 * kPfTrStride * 4;
    static_assert(KS == 1 || kLdsBytes >= kPfWaves * 2 * 8 * 64 * 16, "exchange of two token groups per round");
    __shared__ __attribute__((aligned(16))) char lds_raw[kLdsBytes];
    const int tid = threadIdx.x & (kPfThreads - 1);                     // thread within its half
    const int lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int wave = wave8 & (kPfWaves - 1), grp = wave8 / kPfWaves;
    _Float16 (*const lds_act)[kActBuf] = (_Float16 (*)[kActBuf])lds_raw + 4 * grp;
    const int g = lane >> 4, j = lane & 15;

    // workgroups that share a token tile run on the same XCD (ids are dealt round-robin to the
    // 8 XCDs) so the activation tile is fetched into that XCD's L2 once
    const int total = a.m_tiles * a.n_tiles;
    int id = blockIdx.x;
    {
        const int per = total / 8;
        if (id < per * 8) id = (id & 7) * per + (id >> 3);
    }
    const int m_tile = id / a.n_tiles, n_tile = id - m_tile * a.n_tiles;
    const int split = blockIdx.y;
    // (with KS = 2 the host makes the workgroup's part a multiple of eight steps: equal halves, both
    // multiples of four, so that all eight waves pass the same barriers)
    const int wg_begin = split * a.steps_per_split;
    const int wg_steps = max(0, min(a.nst, wg_begin + a.steps_per_split) - wg_begin);
    const int n_my = wg_steps / KS;
    const int s_begin = wg_begin + grp * n_my;

    int rb = n_tile * kPfWaves + wave;
    const bool rb_valid = rb < a.n_rb;
    if (!rb_valid) rb = a.n_rb - 1;                        // keep loading valid memory, store nothing
    const int m0 = m_tile * kTok;

    // activation tile: 64 (32) tokens x 64 halves = 512 (256) chunks of 16 bytes, 2 (1) per thread:
    // chunk c = tid + 256 i  ->  token c / 8, 16-byte column c % 8
    const int ld_tok = tid >> 3, ld_kc = tid & 7;                       // chunk i adds 32 tokens
    const _Float16* act_ptr = a.act + (size_t)(m0 + ld_tok) * a.lda + (size_t)s_begin * 64 + ld_kc * 8;
    const size_t act_i = (size_t)32 * a.lda;
    const int lds_off = ld_tok * kPfLdsStride + ld_kc * 8;
    const v4u32* w_ptr = (const v4u32*)a.tiles + ((size_t)rb * a.nst + s_begin) * 64 + lane;

    v4f acc[8][TG];
#pragma unroll
    for (int p = 0; p < 8; ++p)
#pragma unroll
        for (int tg = 0; tg < TG; ++tg) acc[p][tg] = v4f{0.f, 0.f, 0.f, 0.f};

    // two register sets for the activation chunks and the tile words: set (s & 1) belongs to step s
    // (named registers, not arrays: arrays that are written under a condition end up in LDS)
    uint4 a00, a01 = {0, 0, 0, 0}, a10, a11 = {0, 0, 0, 0};
    v4u32 wr0, wr1, wr2, wr3 = {0, 0, 0, 0};
#define PF_LOAD_ACT(R, step)                                                             \
    do {                                                                                 \
        const _Float16* q = act_ptr + (size_t)(step) * 64;                               \
        R##0 = *(const uint4*)(q);                                                       \
        if (TG == 4) R##1 = *(const uint4*)(q + act_i);                                  \
    } while (0)
    // (ONES = two fp16 1.0, or zero where the chunks are a re-read past the end of the reduction:
    // the running sums of the thread's chunks, S of its one or two tokens, must see a step once)
#define PF_STORE_ACT(buf, R, ONES)                                                       \
    do {                                                                                 \
        _Float16* q = &lds_act[buf][lds_off];                                            \
        *(uint4*)(q) = R##0;                                                             \
        ssum0 = pf_sum8(R##0, ONES, ssum0);                                              \
        if (TG == 4) {                                                                   \
            *(uint4*)(q + 32 * kPfLdsStride) = R##1;                                     \
            ssum1 = pf_sum8(R##1, ONES, ssum1);                                          \
        }                                                                                \
    } while (0)
    // one reduction step on LDS buffer CUR with tile words W; the planes are kept in program
    // order (scheduling barriers) so that only one expanded operand is alive at a time
    float ssum0 = 0.f, ssum1 = 0.f;
    const half2v ones = {(_Float16)1.0f, (_Float16)1.0f}, none = {(_Float16)0.f, (_Float16)0.f};
    // B operands (activations of the 4 token groups) for one half step: two named register sets
    // (reduction offsets 0..7 or 8..15 of each 16): set p for the first halves, q for the second
    v8h p0, p1, p2 = {}, p3 = {}, q0, q1, q2 = {}, q3 = {};
#define PF_READ_B(R, BUF, H)                                                             \
    do {                                                                                 \
        const _Float16* lr = &lds_act[BUF][j * kPfLdsStride + 16 * g + 8 * (H)];         \
        R##0 = *(const v8h*)(lr);                                                        \
        R##1 = *(const v8h*)(lr + 1 * 16 * kPfLdsStride);                                \
        if (TG == 4) {                                                                   \
            R##2 = *(const v8h*)(lr + 2 * 16 * kPfLdsStride);                            \
            R##3 = *(const v8h*)(lr + 3 * 16 * kPfLdsStride);                            \
        }                                                                                \
    } while (0)
#define PF_MFMA(P, G, B) acc[P][G] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aop, B, acc[P][G], 0, 0, 0)
    // one half step: 8 planes x 4 token groups.  w0 / w1 are the two tile words of this half.
    // The scheduler is asked to alternate one MFMA with one vector op, so that the expansion of
    // the next plane runs in the shadow of the current plane's MFMAs.
    // plane p of a half step: bit p of each 16-bit half of the two tile words and of their copies
    // shifted down by a byte (reduction indices (k0, k2), (k1, k3), (k4, k6), (k5, k7))
#define PF_EXPAND(AU, p, w0, w0s, w1, w1s)                                               \
    do {                                                                                 \
        AU.x = (w0) & (0x00010001u << (p));                                              \
        AU.y = (w0s) & (0x00010001u << (p));                                             \
        AU.z = (w1) & (0x00010001u << (p));                                              \
        AU.w = (w1s) & (0x00010001u << (p));                                             \
    } while (0)
#define PF_HALF(R, w0, w1)                                                               \
    do {                                                                                 \
        uint32_t w0s = (w0) >> 8, w1s = (w1) >> 8;                                       \
        asm volatile("" : "+v"(w0s), "+v"(w1s));        /* one shift per word, not one per plane */ \
        v4u32 au_next;                                                                   \
        PF_EXPAND(au_next, 0, w0, w0s, w1, w1s);                                         \
        __builtin_amdgcn_sched_barrier(0);                                               \
        _Pragma("unroll") for (int p = 0; p < 8; ++p) {                                  \
            const v8h aop = __builtin_bit_cast(v8h, au_next);                            \
            if (p < 7) PF_EXPAND(au_next, p + 1, w0, w0s, w1, w1s);                      \
            PF_MFMA(p, 0, R##0); PF_MFMA(p, 1, R##1);                                    \
            if (TG == 4) { PF_MFMA(p, 2, R##2); PF_MFMA(p, 3, R##3); }                   \
            _Pragma("unroll") for (int i = 0; i < TG; ++i) {                             \
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);        /* 1 MFMA */   \
                __builtin_amdgcn_sched_group_barrier(0x002, 4 / TG, 0);   /* its share of the 4 vector ops */ \
            }                                                                            \
            __builtin_amdgcn_sched_barrier(0);                                           \
        }                                                                                \
    } while (0)

    // byte b of a tile word holds reduction index 4v+b, its bit p the row 16p + lane%16: bit p of
    // the two halves of the word are (k0, k2), of the word shifted down by 8 (k1, k3)
    // n_my is a multiple of 4 (the reduction is padded to 4 steps and so are the splits), and the
    // loop body is branch-free: prefetches past the end re-read the last step instead of being
    // skipped, so no control-flow join forces copies of the 256 accumulator registers.
    // Step s works on LDS buffer s % 4 with tile-word set s % 4; everything it needs was requested
    // well ahead, and every register set has ONE role per position of the four-step body, so the
    // loop carries no register copies:
    //   read the second-half operands of step s | fetch step s+3 from global (activations into the
    //   free one of two register sets, tile words into the set that step s-1 used) | MFMAs of the
    //   first half | write step s+2 (fetched during step s-1) into its buffer | read the
    //   first-half operands of step s+1 (written during step s-1, before the last barrier) | MFMAs
    //   of the second half | barrier.
    // Every LDS read is issued half a step before its first use, every global load one and a half
    // steps (activations) or three (tile words, which come from HBM).  A buffer is overwritten two
    // steps (two barriers) after its last read.
    if (n_my > 0) {
        const int last = n_my - 1;
        // the order in which loads are issued is pinned (scheduling barriers) and is the same in the
        // prologue and in the loop -- activation chunks, then tile words, per step -- so that the
        // compiler can wait for "all but the newest n" loads instead of for all of them
        const int i1 = min(1, last), i2 = min(2, last);
        PF_LOAD_ACT(a0, 0);
        wr0 = w_ptr[0];
        __builtin_amdgcn_sched_barrier(0);
        PF_LOAD_ACT(a1, i1);
        wr1 = w_ptr[(size_t)i1 * 64];
        __builtin_amdgcn_sched_barrier(0);
        PF_STORE_ACT(0, a0, ones);
        PF_STORE_ACT(1, a1, 1 <= last ? ones : none);
        __builtin_amdgcn_sched_barrier(0);
        PF_LOAD_ACT(a1, i2);
        wr2 = w_ptr[(size_t)i2 * 64];
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        PF_READ_B(p, 0, 0);
#define PF_STEP(CUR, NXT, ST, AL, AS, WL, WC, step)                                      \
    do {                                                                                 \
        PF_READ_B(q, CUR, 1);                                                            \
        const int nx = min((step) + 3, last);                                            \
        __builtin_amdgcn_sched_barrier(0);                                               \
        PF_LOAD_ACT(AL, nx);                                                             \
        WL = w_ptr[(size_t)nx * 64];                                                     \
        __builtin_amdgcn_sched_barrier(0);                                               \
        PF_HALF(p, WC.x, WC.y);                                                          \
        PF_STORE_ACT(ST, AS, (step) + 2 <= last ? ones : none);                          \
        PF_READ_B(p, NXT, 0);                                                            \
        PF_HALF(q, WC.z, WC.w);                                                          \
        __syncthreads();                                                                 \
    } while (0)
        for (int s = 0; s < n_my; s += 4) {
            PF_STEP(0, 1, 2, a0, a1, wr3, wr0, s);
            PF_STEP(1, 2, 3, a1, a0, wr0, wr1, s + 1);
            PF_STEP(2, 3, 0, a0, a1, wr1, wr2, s + 2);
            PF_STEP(3, 0, 1, a1, a0, wr2, wr3, s + 3);
        }
#undef PF_STEP
    }
#undef PF_LOAD_ACT
#undef PF_STORE_ACT
#undef PF_HALF
#undef PF_EXPAND
#undef PF_READ_B
#undef PF_MFMA

    // S of the tile's tokens: the eight threads that staged a token's chunks add up their sums
    // (neighbouring lanes), and the sums go through LDS (the activation buffers are done with) to
    // the lanes that hold the token's results
    float* const lds_f = (float*)&lds_raw[0];
    ssum0 += __shfl_xor(ssum0, 1); ssum0 += __shfl_xor(ssum0, 2); ssum0 += __shfl_xor(ssum0, 4);
    if (TG == 4) { ssum1 += __shfl_xor(ssum1, 1); ssum1 += __shfl_xor(ssum1, 2); ssum1 += __shfl_xor(ssum1, 4); }
    __syncthreads();
    if (ld_kc == 0) {
        lds_f[grp * 64 + ld_tok] = ssum0;
        if (TG == 4) lds_f[grp * 64 + ld_tok + 32] = ssum1;
    }
    __syncthreads();
    float s_tok[TG];
#pragma unroll
    for (int tg = 0; tg < TG; ++tg) {
        s_tok[tg] = lds_f[tg * 16 + j];
        if (KS == 2) s_tok[tg] += lds_f[64 + tg * 16 + j];
    }
    __syncthreads();                                       // the sums are read: LDS changes hands once more
    if (KS == 2) {
        // waves 4..7 hand their accumulators to waves 0..3, two token groups per round: a lane's 16
        // registers of a token group go to the same lane of the partner (no transposition here).
        // Every wave adds what it reads (the second half's sums are not used any further): no
        // branch around a write to the accumulators.
        float* const xr = lds_f + wave * (2 * 8 * 64 * 4);
#pragma unroll
        for (int round = 0; round < 2; ++round) {
            if (grp == 1) {
#pragma unroll
                for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                    for (int p = 0; p < 8; ++p) *(v4f*)(xr + ((tl * 8 + p) * 64 + lane) * 4) = acc[p][2 * round + tl];
            }
            __syncthreads();
#pragma unroll
            for (int tl = 0; tl < 2; ++tl)
#pragma unroll
                for (int p = 0; p < 8; ++p) acc[p][2 * round + tl] += *(const v4f*)(xr + ((tl * 8 + p) * 64 + lane) * 4);
            __syncthreads();
        }
        if (grp == 1) return;
    }
    if (!rb_valid) return;

    // Result layout: lane (g, j), register v of acc[p][tg]  <->  C[token m0 + 16 tg + j][row 128 rb + 16 p + 4 g + v],
    // i.e. a lane holds 4 consecutive rows of a token and a store straight from the accumulators
    // would write 64-byte pieces of 16 different output rows.  Each wave therefore turns its
    // results round in a private LDS region, 16 tokens at a time: written in the layout above,
    // read back as [token][128 rows], so that one store instruction covers two tokens x 512
    // contiguous bytes (256 for fp16 T).  Measured on 28672x8192 r=3520 at 2048 tokens: the stores
    // were 18 % of the time of a forward.
    // c = S - 2^(25-p) acc = -(2P - S): the negated signed sum, so every factor below carries a minus
    float* const tr = lds_f + wave * (16 * kPfTrStride);
    const int rd_col = 4 * (lane & 31), rd_tok = lane >> 5;
    const int n0 = rb * kTileRows + rd_col;                 // the 4 rows this lane stores
    const bool aligned_y = (a.n_real & 3) == 0;
    float osc[4] = {0.f, 0.f, 0.f, 0.f};
    if (EPI == EPI_Y && aligned_y && n0 < a.n_real) {
        const uint2 sc = *(const uint2*)(a.out_scale + n0);
        osc[0] = h2f((uint16_t)(sc.x & 0xFFFFu));
        osc[1] = h2f((uint16_t)(sc.x >> 16));
        osc[2] = h2f((uint16_t)(sc.y & 0xFFFFu));
        osc[3] = h2f((uint16_t)(sc.y >> 16));
    }
#pragma unroll
    for (int tg = 0; tg < TG; ++tg) {
        float f = 1.0f;
        if (EPI == EPI_Y) {
            const int tok = m0 + tg * 16 + j;
            f = tok < a.batch ? -a.tok_scale[tok] : 0.f;
        }
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const float w_p = -(float)(1u << (25 - p));
            const v4f r = acc[p][tg];
            v4f c = {fmaf(r.x, w_p, s_tok[tg]), fmaf(r.y, w_p, s_tok[tg]), fmaf(r.z, w_p, s_tok[tg]), fmaf(r.w, w_p, s_tok[tg])};
            if (EPI == EPI_Y) c *= f;
            *(v4f*)(tr + j * kPfTrStride + 16 * p + 4 * g) = c;
        }
        // (the region is private to the wave and a wave's LDS operations complete in order)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int t = rd_tok + 2 * i;
            const int tok = m0 + tg * 16 + t;
            const v4f c = *(const v4f*)(tr + t * kPfTrStride + rd_col);
            if (EPI == EPI_PARTIAL) {
                float* dst = a.partial + ((size_t)split * a.m_pad + tok) * a.n_pad + n0;
                *(v4f*)dst = c;
            } else if (EPI == EPI_T) {
                store_t(a, tok, n0, c);
            } else {
                if (tok < a.batch) {
                    const size_t at = (size_t)tok * a.n_real + n0;
                    const float cv[4] = {c.x, c.y, c.z, c.w};
                    if (aligned_y) {                        // rows stay aligned: one store per lane
                        if (n0 < a.n_real) {
                            v4f o;
                            o.x = cv[0] * osc[0];
                            o.y = cv[1] * osc[1];
                            o.z = cv[2] * osc[2];
                            o.w = cv[3] * osc[3];
                            if (a.y_dtype == NQ_F32) {
                                __builtin_nontemporal_store(o, (v4f*)((float*)a.y_out + at));
                            } else {
                                typedef uint32_t v2u32 __attribute__((ext_vector_type(2)));
                                v2u32 pk;
                                pk.x = (uint32_t)float_to_out16(o.x, a.y_dtype) | ((uint32_t)float_to_out16(o.y, a.y_dtype) << 16);
                                pk.y = (uint32_t)float_to_out16(o.z, a.y_dtype) | ((uint32_t)float_to_out16(o.w, a.y_dtype) << 16);
                                __builtin_nontemporal_store(pk, (v2u32*)((uint16_t*)a.y_out + at));     // (as the fp32 store: written once, not read here)
                            }
                        }
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (n0 + v < a.n_real) store_out(a.y_out, a.y_dtype, at + v, cv[v] * h2f(a.out_scale[n0 + v]));
                    }
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
    }
}

// sum the split-K partials and apply the epilogue; one thread per four consecutive outputs
template <int EPI>
__global__ void __launch_bounds__(256)
prefill_finalize_kernel(GemmArgs a)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int n4 = a.n_pad / 4;
    const size_t total = (size_t)a.m_pad * n4;
    if (idx >= total) return;
    const int tok = (int)(idx / n4), n0 = (int)(idx % n4) * 4;
    v4f c = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < a.splits; ++s) c += *(const v4f*)(a.partial + ((size_t)s * a.m_pad + tok) * a.n_pad + n0);
    if (EPI == EPI_T) {
        store_t(a, tok, n0, c);
    } else {
        if (tok < a.batch) {
            const float f = -a.tok_scale[tok];
            const float cv[4] = {c.x, c.y, c.z, c.w};
            const size_t at = (size_t)tok * a.n_real + n0;
            if ((a.n_real & 3) == 0) {                     // rows stay aligned: one load of scales, one store
                if (n0 < a.n_real) {
                    const uint2 sc = *(const uint2*)(a.out_scale + n0);
                    v4f o;
                    o.x = cv[0] * f * h2f((uint16_t)(sc.x & 0xFFFFu));
                    o.y = cv[1] * f * h2f((uint16_t)(sc.x >> 16));
                    o.z = cv[2] * f * h2f((uint16_t)(sc.y & 0xFFFFu));
                    o.w = cv[3] * f * h2f((uint16_t)(sc.y >> 16));
                    if (a.y_dtype == NQ_F32) {
                        *(v4f*)((float*)a.y_out + at) = o;
                    } else {
                        uint2 pk;
                        pk.x = (uint32_t)float_to_out16(o.x, a.y_dtype) | ((uint32_t)float_to_out16(o.y, a.y_dtype) << 16);
                        pk.y = (uint32_t)float_to_out16(o.z, a.y_dtype) | ((uint32_t)float_to_out16(o.w, a.y_dtype) << 16);
                        *(uint2*)((uint16_t*)a.y_out + at) = pk;
                    }
                }
            } else {
                for (int v = 0; v < 4; ++v)
                    if (n0 + v < a.n_real) store_out(a.y_out, a.y_dtype, at + v, cv[v] * f * h2f(a.out_scale[n0 + v]));
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
static size_t al256(size_t v) { return (v + 255) / 256 * 256; }

struct PfLayout {
    int m_pad, k1, k2, n1_pad, n2_pad;
    int splits1, splits2;
    int tg1, tg2;             // token groups of 16 per workgroup tile of the two GEMMs (4 or 2)
    int ks1, ks2;             // halves of the reduction taken inside a workgroup (1, or 2: eight waves)
    size_t off_x, off_t, off_scale, off_partial, total;
};

// Tiling of one GEMM: token groups per workgroup tile (4 = 64 tokens, 2 = 32 tokens) and the number of
// workgroups the reduction is split over, for outputs that alone give too few workgroups to
// cover the chip.  Cost model in microseconds, constants measured on the 70B MLP shapes (with the
// first version of the kernel; the kernel has since gained a few per cent everywhere, and sweeps
// over splits and tile sizes on those shapes still land on the choices this model makes):
//  - a reduction step of a 64-token workgroup takes 0.73 us when it has its CU to itself and
//    1.17 us when two share one (two is all that fits);
//  - a 32-token workgroup needs 0.60 us per step alone (the sign expansion is not halved), and a
//    CU completes at most 3.9 of their steps per microsecond (up to four fit);
//  - splitting costs a finalize launch (2 us) plus, per split, the write and re-read of one set of
//    fp32 partial sums, not overlapped with anything: about 2.3 MB per microsecond.
// steps per split, rounded up to a multiple of 4 (as nst itself is): the kernel's loop body is four
// steps; of 8 where the workgroup halves its part once more (ks = 2: nst is then a multiple of 8 too)
static int steps_per_split4(int nst, int splits, int ks = 1)
{
    const int per = (nst + splits - 1) / splits, q = 4 * ks;
    return (per + q - 1) / q * q;
}

struct GemmTiling { int tg, splits, ks; };
static GemmTiling choose_tiling(int m_pad, int n_rb, int nst, int n_pad)
{
    const int cus = device_cu_count();
    const int n_tiles = (n_rb + kPfWaves - 1) / kPfWaves;
    const double partial_us = (double)m_pad * n_pad * 4.0 / 2.3e6;
    GemmTiling best = {4, 1, 1};
    double best_cost = 1e30;
    for (int tg = 4; tg >= 2; tg -= 2) {
        const int wgs = (m_pad / (16 * tg)) * n_tiles;
        const int per_cu = tg == 4 ? 2 : 4;
        for (int s = 1; s <= 16; ++s) {
            const int per = steps_per_split4(nst, s);
            if (s > 1 && per < 8) break;
            const int total = wgs * s;
            // 32-token tiles were measured, and pay, only where they let an unsplit GEMM cover the chip
            if (tg == 2 && (s > 1 || total > cus)) break;
            // workgroups per CU in full rounds, then in the last, partial one
            auto step_us = [&](int k) {
                if (tg == 4) return k <= 1 ? 0.73 : 1.17;
                return std::max(0.60, k / 3.9);
            };
            const int full = total / (per_cu * cus), rem = total % (per_cu * cus);
            double cost = (double)full * per * step_us(per_cu);
            if (rem) cost += per * step_us((rem + cus - 1) / cus);
            if (s > 1) cost += 2.0 + s * partial_us;
            if (cost < best_cost) { best_cost = cost; best = {tg, s, 1}; }
        }
    }
    // A long reduction whose 64-token tiles number no more than the CUs and that the model leaves
    // unsplit, or splits no further than into one part per CU: eight-wave workgroups, one per CU,
    // each halving its part of the reduction through LDS -- half the partial sums in memory, or none.
    // Measured on the 70B MLP shapes: gemm 1 of the gate layer at 2048 tokens (224 tiles, 128 steps)
    // 106 -> 99 us, of the down layer (224 tiles, 448 steps, split in two before) 300 -> 284 us
    // including the finalize pass it no longer needs; gate layer at 1024 tokens (112 tiles, two
    // parts per tile) 244 -> 213 us per forward, at 512 tokens (56 tiles, four parts) 115 -> 113 us.
    const int wgs4 = (m_pad / 64) * n_tiles;
    if (best.tg == 4 && wgs4 <= cus && nst % 8 == 0) {
        const int s_fill = std::max(1, cus / wgs4);
        // (a half of at least 16 steps; of 32 where the tile is not split otherwise: 28-step halves of
        // an unsplit second GEMM measured 2 % slower than four-wave workgroups)
        // and parts of equal length (three unequal parts of 128 steps at 768 tokens: 194 against 174 us
        // per forward with four-wave workgroups)
        if (best.splits <= 2 * s_fill && nst % (8 * s_fill) == 0 && nst / (2 * s_fill) >= (s_fill == 1 ? 32 : 16))
            best = {4, s_fill, 2};
    }
    return best;
}

static PfLayout pf_layout(int64_t d_out, int64_t d_in, int64_t r, int batch)
{
    PfLayout L;
    L.m_pad = (int)round_up(batch, kPfTokens);
    L.k1 = (int)n_steps(d_in) * 64;
    L.k2 = (int)n_steps(r) * 64;
    L.n1_pad = (int)n_rowblocks(r) * kTileRows;
    L.n2_pad = (int)n_rowblocks(d_out) * kTileRows;
    const GemmTiling t1 = choose_tiling(L.m_pad, (int)n_rowblocks(r), (int)n_steps(d_in), L.n1_pad);
    const GemmTiling t2 = choose_tiling(L.m_pad, (int)n_rowblocks(d_out), (int)n_steps(r), L.n2_pad);
    L.tg1 = t1.tg; L.splits1 = t1.splits; L.ks1 = t1.ks;
    L.tg2 = t2.tg; L.splits2 = t2.splits; L.ks2 = t2.ks;
    if (opt(OPT_PF_TG1) >= 0) L.tg1 = opt(OPT_PF_TG1) == 2 ? 2 : 4;
    if (opt(OPT_PF_TG2) >= 0) L.tg2 = opt(OPT_PF_TG2) == 2 ? 2 : 4;
    if (opt(OPT_PF_SPLITS1) >= 0) L.splits1 = std::max(1, opt(OPT_PF_SPLITS1));
    if (opt(OPT_PF_SPLITS2) >= 0) L.splits2 = std::max(1, opt(OPT_PF_SPLITS2));
    if (opt(OPT_PF_KS1) >= 0) L.ks1 = opt(OPT_PF_KS1) == 2 ? 2 : 1;
    if (opt(OPT_PF_KS2) >= 0) L.ks2 = opt(OPT_PF_KS2) == 2 ? 2 : 1;
    // the in-workgroup split needs 64-token tiles and a reduction of whole groups of eight steps
    if (L.tg1 != 4 || n_steps(d_in) % 8 != 0) L.ks1 = 1;
    if (L.tg2 != 4 || n_steps(r) % 8 != 0) L.ks2 = 1;
    if (opt_flag(OPT_PF_VERBOSE))
        fprintf(stderr, "prefill tiling B=%d: gemm1 tg=%d splits=%d ks=%d, gemm2 tg=%d splits=%d ks=%d\n", batch, L.tg1, L.splits1,
                L.ks1, L.tg2, L.splits2, L.ks2);
    size_t o = 0;
    L.off_x = o; o += al256((size_t)L.m_pad * L.k1 * 2);
    L.off_t = o; o += al256((size_t)L.m_pad * L.k2 * 2);
    L.off_scale = o; o += al256((size_t)L.m_pad * 4);
    L.off_partial = o;
    size_t p1 = L.splits1 > 1 ? (size_t)L.splits1 * L.m_pad * L.n1_pad * 4 : 0;
    size_t p2 = L.splits2 > 1 ? (size_t)L.splits2 * L.m_pad * L.n2_pad * 4 : 0;
    o += al256(std::max(p1, p2));
    L.total = o;
    return L;
}

size_t prefill_workspace_bytes(int64_t d_out, int64_t d_in, int64_t r, int batch)
{
    return pf_layout(d_out, d_in, r, batch).total;
}

// columns [c0, c1) of every row of a [rows][ld] fp16 matrix := 0
__global__ void __launch_bounds__(256)
prefill_zero_cols_kernel(_Float16* __restrict__ m, int ld, int c0, int c1, int rows)
{
    const int w = c1 - c0;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)rows * w) return;
    const int row = (int)(idx / w), col = c0 + (int)(idx % w);
    m[(size_t)row * ld + col] = (_Float16)0.f;
}

template <int EPI>
static int run_gemm(const GemmArgs& a, int tg, int ks, hipStream_t s)
{
    dim3 grid(a.m_tiles * a.n_tiles, a.splits);
    if (ks == 2 && (tg != 4 || a.nst % 8 != 0 || a.steps_per_split % 8 != 0)) {
        set_error("prefill: the in-workgroup split needs 64-token tiles and parts of whole groups of eight steps");
        return NQ_E_INVALID_ARG;
    }
    if (a.splits > 1) {
        if (ks == 2) hipLaunchKernelGGL((prefill_gemm_kernel<EPI_PARTIAL, 4, 2>), grid, dim3(2 * kPfThreads), 0, s, a);
        else if (tg == 4) hipLaunchKernelGGL((prefill_gemm_kernel<EPI_PARTIAL, 4>), grid, dim3(kPfThreads), 0, s, a);
        else hipLaunchKernelGGL((prefill_gemm_kernel<EPI_PARTIAL, 2>), grid, dim3(kPfThreads), 0, s, a);
        NQ_HIP(hipGetLastError());
        const size_t total = (size_t)a.m_pad * (a.n_pad / 4);
        hipLaunchKernelGGL((prefill_finalize_kernel<EPI>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a);
    } else {
        if (ks == 2) hipLaunchKernelGGL((prefill_gemm_kernel<EPI, 4, 2>), grid, dim3(2 * kPfThreads), 0, s, a);
        else if (tg == 4) hipLaunchKernelGGL((prefill_gemm_kernel<EPI, 4>), grid, dim3(kPfThreads), 0, s, a);
        else hipLaunchKernelGGL((prefill_gemm_kernel<EPI, 2>), grid, dim3(kPfThreads), 0, s, a);
    }
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

int launch_prefill(const PrefillArgs& p, hipStream_t s)
{
    const PfLayout L = pf_layout(p.d_out, p.d_in, p.r, p.batch);
    char* ws = (char*)p.workspace;
    _Float16* xs = (_Float16*)(ws + L.off_x);
    _Float16* t = (_Float16*)(ws + L.off_t);
    float* tok_scale = (float*)(ws + L.off_scale);
    float* partial = (float*)(ws + L.off_partial);
    // |x''| < 2^13, so |t''| < d_in * 2^13; g brings that to <= 2^15 (fp16 range 65504)
    int lg = 0;
    while (((int64_t)1 << lg) < p.d_in) ++lg;
    // (with a rank-wise scale, |s_mid| <= 2^mid_exp, T = X''V g s_mid stays within the same bound)
    const float g_t = ldexpf(1.0f, -(lg > 2 ? lg - 2 : 0) - (p.s_mid ? p.mid_exp : 0));

    if (p.x_dtype == NQ_F32)
        hipLaunchKernelGGL(prefill_prescale_kernel<NQ_F32>, dim3(p.batch), dim3(kPreThreads), 0, s, p.x, p.s_in, (int)p.d_in,
                           L.k1, g_t, xs, tok_scale);
    else if (p.x_dtype == NQ_F16)
        hipLaunchKernelGGL(prefill_prescale_kernel<NQ_F16>, dim3(p.batch), dim3(kPreThreads), 0, s, p.x, p.s_in, (int)p.d_in,
                           L.k1, g_t, xs, tok_scale);
    else
        hipLaunchKernelGGL(prefill_prescale_kernel<NQ_BF16>, dim3(p.batch), dim3(kPreThreads), 0, s, p.x, p.s_in, (int)p.d_in,
                           L.k1, g_t, xs, tok_scale);
    NQ_HIP(hipGetLastError());

    GemmArgs a{};
    a.m_pad = L.m_pad;
    a.batch = p.batch;
    a.partial = partial;
    // gemm1: T = X'' V
    a.act = xs; a.lda = L.k1; a.tiles = p.vt_tiles;
    a.t_out = t; a.ldt = L.k2; a.t_scale = g_t; a.mid_scale = p.s_mid;
    a.n_real = (int)p.r; a.n_rb = (int)n_rowblocks(p.r); a.nst = (int)n_steps(p.d_in);
    a.n_tiles = (a.n_rb + kPfWaves - 1) / kPfWaves;
    a.splits = L.splits1; a.steps_per_split = steps_per_split4(a.nst, a.splits, L.ks1);
    a.n_pad = L.n1_pad;
    a.m_tiles = L.m_pad / (16 * L.tg1);
    int rc = run_gemm<EPI_T>(a, L.tg1, L.ks1, s);
    if (rc != NQ_OK) return rc;
    if (L.k2 > L.n1_pad) {
        // columns of T beyond the last 128-row block of gemm1 are padding of gemm2's reduction:
        // they must be exact zeros (the padded sign bits expand to -1, not to 0)
        const size_t cnt = (size_t)L.m_pad * (L.k2 - L.n1_pad);
        hipLaunchKernelGGL(prefill_zero_cols_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, s, t, L.k2,
                           L.n1_pad, L.k2, L.m_pad);
        NQ_HIP(hipGetLastError());
    }
    // gemm2: y = T U^T
    a.act = t; a.lda = L.k2; a.tiles = p.u_tiles;
    a.y_out = p.y; a.y_dtype = p.y_dtype; a.tok_scale = tok_scale; a.out_scale = p.s_out;
    a.n_real = (int)p.d_out; a.n_rb = (int)n_rowblocks(p.d_out); a.nst = (int)n_steps(p.r);
    a.n_tiles = (a.n_rb + kPfWaves - 1) / kPfWaves;
    a.splits = L.splits2; a.steps_per_split = steps_per_split4(a.nst, a.splits, L.ks2);
    a.n_pad = L.n2_pad;
    a.m_tiles = L.m_pad / (16 * L.tg2);
    return run_gemm<EPI_Y>(a, L.tg2, L.ks2, s);
}

}  // namespace nq
