// Device-side helpers shared by the kernel files of libnq_binlr (not installed): vector types,
// 16-bit float decoding, the fixed-point split of a chunk of activations, tile loads and the
// one-step multiply-accumulate of the streaming kernels (Section 3.1 Eq. 1 evaluated as two
// sign-matrix x vector products; Appendix E.2).
#pragma once
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

typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) v4u* gptr_v4u;    // global (not generic) address space
typedef const __attribute__((address_space(1))) v4f* gptr_v4f;
typedef const __attribute__((address_space(1))) uint16_t* gptr_u16;

// chunk c (16 consecutive elements) of token row `base` of the vector d describes, times its scale
__device__ inline void load_chunk16(const QuantDesc& d, int64_t base, int c, bool vec, float v[16])
{
    const int j0 = c * 16;
    if (vec && j0 + 16 <= d.N) {
        // the scales are requested before the (type-dependent) loads of x, so that both are in flight together
        v4u sraw[2] = {v4u{0, 0, 0, 0}, v4u{0, 0, 0, 0}};
        if (d.scale) {
            const gptr_v4u sp = (gptr_v4u)(d.scale + j0);
            sraw[0] = sp[0];
            sraw[1] = sp[1];
        }
        if (d.dtype == NQ_F32) {
            // (global, not generic, address space: plain vector loads, exact wait counts)
            const gptr_v4f p = (gptr_v4f)((const float*)d.x + base + j0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const v4f f = p[q];
                v[4 * q] = f.x; v[4 * q + 1] = f.y; v[4 * q + 2] = f.z; v[4 * q + 3] = f.w;
            }
        } else {
            const gptr_v4u p = (gptr_v4u)((const uint16_t*)d.x + base + j0);
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const v4u u = p[q];
                uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    uint16_t lo = (uint16_t)(w[i] & 0xFFFFu), hi = (uint16_t)(w[i] >> 16);
                    v[8 * q + 2 * i] = d.dtype == NQ_F16 ? half_bits_to_float(lo) : bf16_bits_to_float(lo);
                    v[8 * q + 2 * i + 1] = d.dtype == NQ_F16 ? half_bits_to_float(hi) : bf16_bits_to_float(hi);
                }
            }
        }
        if (d.scale) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const v4u u = sraw[q];
                uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    v[8 * q + 2 * i] *= half_bits_to_float((uint16_t)(w[i] & 0xFFFFu));
                    v[8 * q + 2 * i + 1] *= half_bits_to_float((uint16_t)(w[i] >> 16));
                }
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int j = j0 + i;
            float f = 0.f;                                  // padding beyond N contributes nothing
            if (j < d.N) {
                f = load_as_float(d.x, d.dtype, base + j);
                if (d.scale) f *= half_bits_to_float(d.scale[j]);
            }
            v[i] = f;
        }
    }
}

// byte 0 of a, b, c, d -> one word (a lowest): three byte-permute instructions
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    const uint32_t ab = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);      // bytes: a.0, b.0, 0, 0
    const uint32_t cd = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(cd, ab, 0x05040100u);                 // ab.0, ab.1, cd.0, cd.1
}

// q = 65536 hi + 256 mid + lo with signed bytes: lo is the (sign-extended) low byte of q,
// mid that of q1 = (q - lo) / 256 = (q + 128) >> 8, hi = (q1 + 128) >> 8; only the low bytes are kept
template <bool STREAMED = false>
__device__ inline long long quantize_chunk16(const float v[16], float inv_step, bool bad, uint4* dst)
{
    uint32_t hi[4], mid[4], lo[4];
    int sum = 0;                                            // |q| <= 2^22, 16 of them: fits
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint32_t q0[4], q1[4], q2[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = bad ? 0 : (int)rintf(v[4 * w + i] * inv_step);
            sum += q;
            const int m = (q + 128) >> 8;
            q0[i] = (uint32_t)q;
            q1[i] = (uint32_t)m;
            q2[i] = (uint32_t)((m + 128) >> 8);
        }
        lo[w] = pack_low_bytes(q0[0], q0[1], q0[2], q0[3]);
        mid[w] = pack_low_bytes(q1[0], q1[1], q1[2], q1[3]);
        hi[w] = pack_low_bytes(q2[0], q2[1], q2[2], q2[3]);
    }
    // the three slices of a chunk sit 4 pieces apart (see bq_piece): consecutive threads = consecutive
    // chunks of a step fill whole 64-byte lines with each of the three stores
    if (STREAMED) {
        // a buffer in global memory that the next launch reads: written around the cache
        typedef __attribute__((address_space(1))) v4u* gptr_wv4u;
        __builtin_nontemporal_store(v4u{hi[0], hi[1], hi[2], hi[3]}, (gptr_wv4u)dst);
        __builtin_nontemporal_store(v4u{mid[0], mid[1], mid[2], mid[3]}, (gptr_wv4u)dst + 4);
        __builtin_nontemporal_store(v4u{lo[0], lo[1], lo[2], lo[3]}, (gptr_wv4u)dst + 8);
    } else {
        dst[0] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        dst[4] = make_uint4(mid[0], mid[1], mid[2], mid[3]);
        dst[8] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    }
    return sum;
}

// sign tiles are streamed once, never reused: keep them from displacing the (reused) activations
__device__ __forceinline__ v4u load_tile_words(const char* base, uint32_t off)
{
    return __builtin_nontemporal_load((gptr_v4u)(base + off));
}
__device__ __forceinline__ v4u load_global_v4u(const char* base, uint32_t off) { return *(gptr_v4u)(base + off); }

// one 64-column step of a token's quantised vector: [3 slices][4 chunks][16 signed bytes]
constexpr uint32_t kBqStepBytes = 4 * kSlices * 16;

// one 64-column step: eight bit planes, each one AND per register and one MFMA per column group
template <int NB>
__device__ __forceinline__ void mac_tile(v4i (&acc)[NB][8], const v4u w, const v4u (&b)[NB])
{
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const uint32_t mask = 0x01010101u << p;
        const v4i a = (v4i)(w & mask);
#pragma unroll
        for (int cg = 0; cg < NB; ++cg)
            acc[cg][p] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, (v4i)b[cg], acc[cg][p], 0, 0, 0);
    }
}

}  // namespace nq
