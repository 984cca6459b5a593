// Measurement aids: what this GPU attains on the two resources the roofline figures are priced
// against -- a plain streaming read of HBM, and a register-resident loop of matrix-core
// instructions.  No part of the forward path; bench.py reports them beside the nominal peaks.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "nq_binlr.h"
#include "nq_internal.h"

namespace nq {

typedef unsigned int pv4u __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) pv4u* gptr_pv4u;
typedef _Float16 pv8h __attribute__((ext_vector_type(8)));
typedef float pv4f __attribute__((ext_vector_type(4)));
typedef int pv4i __attribute__((ext_vector_type(4)));

// Every wave reads its own contiguous share of the buffer in 1 KiB pieces, eight loads in flight,
// non-temporal (the way the stage kernels read their sign tiles); eight waves per SIMD.  (Of the
// variants tried -- shares interleaved between the waves, 4 / 16 loads in flight, cached loads,
// 1 to 16 workgroups per CU -- this one reads fastest.)  The xor of what was read is stored only
// if it hits a value it cannot have, which keeps the loads alive without a write stream.
constexpr int kProbeDepth = 8;
__global__ void __launch_bounds__(256)
probe_read_kernel(const uint32_t* __restrict__ p, size_t pieces_per_wave, uint32_t* __restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const gptr_pv4u base = (gptr_pv4u)p + wave * pieces_per_wave * 64 + lane;
    pv4u acc = {0, 0, 0, 0};
    pv4u buf[kProbeDepth];
    // pieces_per_wave is a multiple of the depth (the host rounds): no branch around a load, so the
    // waits inside the loop stay partial
#pragma unroll
    for (int k = 0; k < kProbeDepth; ++k) buf[k] = __builtin_nontemporal_load(base + k * 64);
    for (size_t c0 = kProbeDepth; c0 < pieces_per_wave; c0 += kProbeDepth) {
#pragma unroll
        for (int k = 0; k < kProbeDepth; ++k) {
            acc ^= buf[k];
            buf[k] = __builtin_nontemporal_load(base + (c0 + k) * 64);
        }
    }
#pragma unroll
    for (int k = 0; k < kProbeDepth; ++k) acc ^= buf[k];
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) sink[wave * 64 + lane] = acc.x;
}

// 16 independent accumulator tiles per wave, two waves per SIMD: nothing but matrix instructions.
template <bool I8>
__global__ void __launch_bounds__(256) probe_mfma_kernel(float* __restrict__ sink, int iters)
{
    pv4f accf[16];
    pv4i acci[16];
    for (int i = 0; i < 16; ++i) {
        accf[i] = pv4f{0, 0, 0, 0};
        acci[i] = pv4i{0, 0, 0, 0};
    }
    pv8h a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(threadIdx.x * 0.001f + i);
        b[i] = (_Float16)(1.0f + i * 0.5f);
    }
    const pv4i ai = {(int)threadIdx.x, 3, 5, 7}, bi = {1, 2, (int)threadIdx.x, 4};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (I8) acci[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ai, bi, acci[i], 0, 0, 0);
            else accf[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, accf[i], 0, 0, 0);
        }
    }
    float s = 0.f;
    for (int i = 0; i < 16; ++i) s += I8 ? (float)(acci[i].x + acci[i].y) : accf[i].x + accf[i].y;
    if (s == 123.456f) sink[threadIdx.x] = s;
}

typedef double pv4d __attribute__((ext_vector_type(4)));

// The same loop with the binary64 instruction (16 x 16 x 4, 2048 operations each): eight accumulators held in named
// variables (as an array the compiler shuttled them between the two register files every iteration).
__global__ __launch_bounds__(256) void probe_mfma_f64_kernel(float* sink, int iters)
{
    pv4d c0 = {0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0, c4 = c0, c5 = c0, c6 = c0, c7 = c0;
    const double a0 = threadIdx.x * 0.001 + 1.0, a1 = a0 + 1.0, b0 = 1.0 + threadIdx.x * 0.5, b1 = b0 + 2.0;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int rep = 0; rep < 2; ++rep) {
            c0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, c3, 0, 0, 0);
            c4 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, c4, 0, 0, 0);
            c5 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, c5, 0, 0, 0);
            c6 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, c6, 0, 0, 0);
            c7 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, c7, 0, 0, 0);
        }
    }
    const pv4d t = ((c0 + c1) + (c2 + c3)) + ((c4 + c5) + (c6 + c7));
    const double s = t.x + t.y;
    if (s == 123.456) sink[threadIdx.x] = (float)s;
}

}  // namespace nq

using namespace nq;

static int fail(int code, const char* msg)
{
    set_error(msg);
    return code;
}

#define PROBE_HIP(call)                                                    \
    do {                                                                   \
        hipError_t e__ = (call);                                           \
        if (e__ != hipSuccess) {                                           \
            rc = hip_fail(e__, #call, __FILE__, __LINE__);                 \
            goto done;                                                     \
        }                                                                  \
    } while (0)

extern "C" int nq_probe_hbm_read(size_t bytes, int iters, int prewarm_ms, double* gb_per_s)
{
    if (!gb_per_s) return fail(NQ_E_NULL, "nq_probe_hbm_read: NULL result pointer");
    if (bytes < ((size_t)64 << 20) || iters < 1 || prewarm_ms < 0 || prewarm_ms > 1000)
        return fail(NQ_E_INVALID_ARG, "nq_probe_hbm_read: at least 64 MiB, one pass, 0..1000 ms of untimed load");
    int rc = NQ_OK;
    uint32_t* buf = nullptr;
    uint32_t* sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    const int blocks = device_cu_count() * 8;
    const size_t per_wave = bytes / 1024 / ((size_t)blocks * 4) / kProbeDepth * kProbeDepth;   // whole rings of pieces per wave
    const size_t n_pieces = per_wave * blocks * 4;
    float ms = 0.f;
    if (per_wave < 1) return fail(NQ_E_INVALID_ARG, "nq_probe_hbm_read: buffer too small for eight pieces per wave");
    PROBE_HIP(hipMalloc((void**)&buf, n_pieces * 1024));
    PROBE_HIP(hipMalloc((void**)&sink, (size_t)blocks * 256 * 4));
    PROBE_HIP(hipMemset(buf, 1, n_pieces * 1024));
    PROBE_HIP(hipEventCreate(&e0));
    PROBE_HIP(hipEventCreate(&e1));
    // untimed passes first (one, plus about prewarm_ms at 5 GB per millisecond)
    for (int i = 0; i < 1 + (int)((double)prewarm_ms * 5.0e9 / (double)(n_pieces * 1024)); ++i)
        hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, nullptr, buf, per_wave, sink);
    PROBE_HIP(hipEventRecord(e0, nullptr));
    for (int i = 0; i < iters; ++i)
        hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, nullptr, buf, per_wave, sink);
    PROBE_HIP(hipEventRecord(e1, nullptr));
    PROBE_HIP(hipEventSynchronize(e1));
    PROBE_HIP(hipGetLastError());
    PROBE_HIP(hipEventElapsedTime(&ms, e0, e1));
    *gb_per_s = (double)n_pieces * 1024.0 * iters / (ms * 1e-3) / 1e9;
done:
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (buf) (void)hipFree(buf);
    if (sink) (void)hipFree(sink);
    return rc;
}

extern "C" int nq_probe_mfma(int dtype, double* tera_ops_per_s)
{
    if (!tera_ops_per_s) return fail(NQ_E_NULL, "nq_probe_mfma: NULL result pointer");
    if (dtype != NQ_F16 && dtype != NQ_I8 && dtype != NQ_F64) return fail(NQ_E_INVALID_ARG, "nq_probe_mfma: dtype must be NQ_F16, NQ_I8 or NQ_F64");
    int rc = NQ_OK;
    float* sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    const int iters = dtype == NQ_F64 ? 1000 : 4000, reps = 3;
    const int blocks = device_cu_count() * 2;                 // 4 waves each: two waves per SIMD
    float ms = 0.f;
    // one instruction = 16 x 16 x K multiply-adds, K = 32 (fp16) or 64 (int8)
    const double ops_per_launch = (double)blocks * 4 * iters * 16 * (dtype == NQ_F16 ? 16384.0 : dtype == NQ_I8 ? 32768.0 : 2048.0);
    PROBE_HIP(hipMalloc((void**)&sink, 256 * 4));
    PROBE_HIP(hipEventCreate(&e0));
    PROBE_HIP(hipEventCreate(&e1));
    for (int i = 0; i < reps + 1; ++i) {
        if (i == 1) PROBE_HIP(hipEventRecord(e0, nullptr));
        if (dtype == NQ_F64) hipLaunchKernelGGL(probe_mfma_f64_kernel, dim3(blocks), dim3(256), 0, nullptr, sink, iters);
        else if (dtype == NQ_F16) hipLaunchKernelGGL(probe_mfma_kernel<false>, dim3(blocks), dim3(256), 0, nullptr, sink, iters);
        else hipLaunchKernelGGL(probe_mfma_kernel<true>, dim3(blocks), dim3(256), 0, nullptr, sink, iters);
    }
    PROBE_HIP(hipEventRecord(e1, nullptr));
    PROBE_HIP(hipEventSynchronize(e1));
    PROBE_HIP(hipGetLastError());
    PROBE_HIP(hipEventElapsedTime(&ms, e0, e1));
    *tera_ops_per_s = ops_per_launch * reps / (ms * 1e-3) / 1e12;
done:
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    return rc;
}
