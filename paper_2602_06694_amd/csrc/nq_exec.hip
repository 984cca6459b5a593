// Dependent layers in ONE launch: a decoder block (or a stack of them) run level by level
// (q, k, v | o | gate, up | down -- the seven projections of Appendix D.3's figure, in the order the
// decode harness of Appendix D.1 calls them) by a persistent grid, batch 1.
//
// A layer forward is two sign-matrix x vector products (Section 3.1 Eq. 1; Appendix E.2), so a
// stack of L levels is 2 L phases, each depending on ALL outputs of the one before.  Run as
// launches, a phase costs a launch-to-launch latency (about 7 us measured) for well under 1 us of
// streaming.  Here one workgroup of 8 waves sits on every CU and walks its own list of tasks; a
// task is a run of 128-row blocks of one phase's sign matrix.  Nothing is ever waited for except data:
//
//  - every value that crosses from one phase to the next (t of stage 1; y where a later layer of
//    the same call reads it) is stored as a 64-bit pair (fp32 bits, epoch) with ONE device-scope
//    store, and read with device-scope loads; a consumer accepts a pair only if it carries the
//    epoch of this launch, else it reads again.  A pair is written by a single 8-byte store, so it
//    is seen whole or not at all: no flag, no counter, no fence, no ordering between stores.  The
//    epoch lives in device memory and is advanced by the last workgroup to leave, so a replay of a
//    captured launch gets a fresh one.
//  - every wait is bounded by a wall-clock limit; a workgroup that gives up sets an error word
//    and leaves, the others see the word (or run into their own limit) and leave too: the grid
//    always drains.
//  - a workgroup requests the first sign tiles of its next task BEFORE it waits for that task's
//    input, so the weights stream while the dependency chain is being walked.
//
// The arithmetic is that of the streaming kernels element for element (same fixed-point split, same
// exact integer sums, same single roundings), so results are bit-identical to a sequence of
// nq_binlr_forward calls.
#include <algorithm>
#include <mutex>
#include <type_traits>
#include <vector>

#include "nq_internal.h"
#include "nq_device.h"

namespace nq {

constexpr int kExecWaves = 8;                      // two per SIMD
constexpr int kExecThreads = 64 * kExecWaves;
constexpr int kExecRing = 8;                       // sign tiles a wave keeps in flight
constexpr int kExecMaxSteps = 512;                 // longest reduction: 32768 elements (96 KiB of LDS as fixed point)
constexpr int kExecEpiInts = 3 * kTileRows;        // per wave: the three slice columns x 128 rows
constexpr int kExecHeld = 4;                       // 16-element chunks of the input a thread keeps in registers (4 x 512 threads x 16 = 32768 elements)

// One task of one workgroup: a run of row blocks of one stage of one layer, with everything the
// kernel needs to know about that stage in the record itself -- a workgroup's records are
// consecutive in memory, so the next one is a neighbouring cache line, requested a task ahead.
// W = 1 << wl waves share a row block, 8 / W row blocks are worked on side by side.
struct ExecTask {
    const uint32_t* tiles;          // sign tiles of A (V^T or U)
    const void* in;                 // the input vector: plain elements of in_dtype (in_ll 0), pairs (1), or none: the LDS array (2)
    const uint16_t* in_scale;       // fp16 [N] or nullptr
    const uint16_t* out_scale;      // fp16 [M rounded up to whole row blocks] or nullptr
    void* out;                      // plain output [M] of out_dtype, or nullptr
    unsigned long long* out_ll;     // pairs [M] for the stages that read this output in the same launch, or nullptr
    int M, N, n_steps, in_dtype, out_dtype, in_ll;
    int rb0, n_rb, wl;
    int out_lds;                    // the (fp32) output also goes to the workgroup's LDS array, for its next task (in_ll == 2)
    int pad[2];
};
static_assert(sizeof(ExecTask) == 96, "task record");

struct ExecState {                  // device words shared by the launches of one executor
    unsigned int epoch;             // of the NEXT launch (never 0: a cleared pair is never valid)
    unsigned int done;              // workgroups of the running launch that have left
    int error;                      // sticky: a wait ran into its limit
    int pad;
};

typedef __attribute__((address_space(1))) unsigned long long* gptr_u64;


__device__ __forceinline__ void ll_store(unsigned long long* p, float v, unsigned int epoch)
{
    const unsigned long long pair = (unsigned long long)__builtin_bit_cast(unsigned int, v) | ((unsigned long long)epoch << 32);
    // (global, not generic, address space: a flat store would count on both wait counters)
    __hip_atomic_store((gptr_u64)p, pair, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Reductions over a wavefront on the data-parallel-primitive path of the vector unit (no LDS traffic):
// quad exchanges, mirrored halves of a 16-lane row, then the four rows through scalar registers.
// The result is the same in every lane.
template <class T, class Op>
__device__ __forceinline__ T wave_reduce32(T v, Op op)
{
    static_assert(sizeof(T) == 4, "32-bit values");
    auto dpp = [](T x, auto ctrl) {
        return __builtin_bit_cast(T, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    v = op(v, dpp(v, std::integral_constant<int, 0xB1>{}));      // quad_perm [1, 0, 3, 2]
    v = op(v, dpp(v, std::integral_constant<int, 0x4E>{}));      // quad_perm [2, 3, 0, 1]
    v = op(v, dpp(v, std::integral_constant<int, 0x141>{}));     // row_half_mirror
    v = op(v, dpp(v, std::integral_constant<int, 0x140>{}));     // row_mirror
    const int b = __builtin_bit_cast(int, v);
    const T r0 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(b, 0)), r1 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(b, 16));
    const T r2 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(b, 32)), r3 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(b, 48));
    return op(op(r0, r1), op(r2, r3));
}

// sum of a 64-bit integer over the wavefront (the halves travel separately, the additions are 64-bit)
__device__ __forceinline__ long long wave_sum64(long long v)
{
    auto dpp = [](long long x, auto ctrl) {
        const int lo = __builtin_amdgcn_mov_dpp((int)(unsigned int)(unsigned long long)x, decltype(ctrl)::value, 0xf, 0xf, true);
        const int hi = __builtin_amdgcn_mov_dpp((int)(unsigned int)((unsigned long long)x >> 32), decltype(ctrl)::value, 0xf, 0xf, true);
        return (long long)(((unsigned long long)(unsigned int)hi << 32) | (unsigned int)lo);
    };
    v += dpp(v, std::integral_constant<int, 0xB1>{});
    v += dpp(v, std::integral_constant<int, 0x4E>{});
    v += dpp(v, std::integral_constant<int, 0x141>{});
    v += dpp(v, std::integral_constant<int, 0x140>{});
    long long t = 0;
#pragma unroll
    for (int r = 0; r < 64; r += 16) {
        const unsigned int lo = (unsigned int)__builtin_amdgcn_readlane((int)(unsigned int)(unsigned long long)v, r);
        const unsigned int hi = (unsigned int)__builtin_amdgcn_readlane((int)(unsigned int)((unsigned long long)v >> 32), r);
        t += (long long)(((unsigned long long)hi << 32) | lo);
    }
    return t;
}

// ---------------------------------------------------------------------------------------------
// LDS: [bq_bytes] the task's input as fixed point (layout of the global buffers of the streaming
// kernels) | [8][3][128] raw sums of the waves | sum of q, largest magnitude, flags
// ---------------------------------------------------------------------------------------------
// tasks[ti .. t_end) of this workgroup; state == nullptr: a lone workgroup whose tasks hand over through LDS only
__device__ __forceinline__ void exec_body(const ExecTask* __restrict__ tasks, int ti, const int t_end,
                                          ExecState* __restrict__ state, int bq_bytes, unsigned long long spin_ticks)
{
    extern __shared__ __align__(16) int lds[];
    constexpr int D = kExecRing;
    char* const lds_bq = (char*)lds;
    int* const lds_epi = (int*)(lds_bq + bq_bytes);
    // reductions over the workgroup go through LDS atomics (one instruction per wave each, no shuffle
    // chains): the sum of the quantised values, the largest magnitude (as the bits of a non-negative
    // float), "a value is not finite", "a wait gave up"
    unsigned long long* const lds_sum = (unsigned long long*)(lds_epi + kExecWaves * kExecEpiInts);
    unsigned int* const lds_max = (unsigned int*)(lds_sum + 1);
    int* const lds_bad = (int*)(lds_max + 1);
    int* const lds_abort = lds_bad + 1;
    float* const lds_t = (float*)(lds_sum + 4);             // (past the 32 bytes of words above) an output kept in LDS for the next task of this workgroup

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, n = lane & 15;
    const unsigned int epoch = state ? state->epoch : 0u;   // written by the previous launch (or the host)
    if (tid == 0) {
        *lds_abort = 0;
        *lds_sum = 0;
        *lds_max = 0;
        *lds_bad = 0;
    }
    __syncthreads();

    v4u wbuf[D];
    // the wave's tile stream of one (task, group of row blocks)
    const char* a_base = nullptr;
    uint32_t a_off = 0;
    int cnt = 0, part = 0, w_of = 1;
    // requests the first D tiles of group `grp` of task `t` (branch-free: a short share re-reads its last tile)
#define NQ_PRIME(t, grp)                                                                           \
    do {                                                                                           \
        const int nst_ = (t).n_steps;                                                      \
        const int wl_ = (t).wl;                                                                    \
        const int sub_ = wave >> wl_;                                                              \
        part = wave - (sub_ << wl_);                                                               \
        w_of = 1 << wl_;                                                                           \
        const int rb_ = (t).rb0 + (grp) * (kExecWaves >> wl_) + sub_;                              \
        const bool act_ = rb_ < (t).rb0 + (t).n_rb;                                                \
        cnt = act_ ? (nst_ - part + w_of - 1) >> wl_ : 0;                                          \
        cnt = cnt < 0 ? 0 : cnt;                                                                   \
        a_base = (const char*)(t).tiles +                                                  \
                 (size_t)(act_ ? rb_ : (t).rb0) * nst_ * (kTileWords * 4);                         \
        a_off = (uint32_t)((cnt > 0 ? part : 0) * 1024 + lane * 16);                               \
        _Pragma("unroll") for (int k = 0; k < D; ++k) {                                            \
            const int kk = k < cnt ? k : (cnt > 0 ? cnt - 1 : 0);                                  \
            wbuf[k] = load_tile_words(a_base, a_off + (uint32_t)kk * (uint32_t)(w_of * 1024));     \
        }                                                                                          \
        a_off += (uint32_t)(D * w_of * 1024);                                                      \
    } while (0)

    // With the first tiles of a task go the scales it will need (static data, usually cold in the caches:
    // a round trip to memory each): the input scales of the chunk this thread owns -- where the input is
    // handed over by another stage and fits one chunk per thread -- and the output scales of the rows this
    // thread finishes in the task's first group.  All of them are requested before the task's input is
    // waited for and converted only when they are used.
    v4u sraw[kExecHeld][2];
#pragma unroll
    for (int c = 0; c < kExecHeld; ++c) sraw[c][0] = sraw[c][1] = v4u{0, 0, 0, 0};
    uint16_t ps[2] = {0, 0};
#define NQ_PREFETCH_SCALES(t)                                                                      \
    do {                                                                                           \
        const uint16_t* const is_ = (t).in_scale;                                                  \
        const int n_ = (t).N;                                                                      \
        _Pragma("unroll") for (int c_ = 0; c_ < kExecHeld; ++c_) {                                 \
            const int j_ = (tid + c_ * kExecThreads) * 16;                                         \
            if (is_ && (t).in_ll && j_ + 16 <= n_) {                                               \
                const gptr_v4u sp_ = (gptr_v4u)(is_ + j_);                                         \
                sraw[c_][0] = sp_[0];                                                              \
                sraw[c_][1] = sp_[1];                                                              \
            }                                                                                      \
        }                                                                                          \
        const uint16_t* const os_ = (t).out_scale;                                         \
        const int per_ = kExecWaves >> (t).wl;                                                     \
        _Pragma("unroll") for (int u = 0; u < 2; ++u) {                                            \
            const int idx_ = tid + u * kExecThreads;                                               \
            const int rb_ = (t).rb0 + (idx_ >> 7);                                                 \
            if (os_ && idx_ < per_ * kTileRows && rb_ < (t).rb0 + (t).n_rb)                        \
                ps[u] = ((gptr_u16)os_)[rb_ * kTileRows + (idx_ & 127)];                           \
        }                                                                                          \
    } while (0)

    ExecTask tk{};
    if (ti < t_end) {
        tk = tasks[ti];
        NQ_PRIME(tk, 0);
        NQ_PREFETCH_SCALES(tk);
    }

    while (ti < t_end) {
        const ExecTask& op = tk;                            // (wave-uniform: the record came through scalar loads)
        // the next record is requested now, a whole task before its fields are needed
        ExecTask nxt = tk;
        const bool more = ti + 1 < t_end;
        if (more) nxt = tasks[ti + 1];
        const int nst = op.n_steps;
        const int n_chunks = 4 * nst;

        // ---- the task's input: load (waiting for this launch's epoch where another stage writes it), scale, quantise ----
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)op.in, 0, op.in_ll ? ((op.N + 1) & ~1) * 8 : 0, 0x00020000);   // (whole 16-byte loads; the arrays are padded)
        QuantDesc qd;
        qd.x = op.in; qd.scale = op.in_scale; qd.bq = nullptr; qd.meta = nullptr;
        qd.N = op.N; qd.n_chunks = n_chunks; qd.x_stride = op.N; qd.dtype = op.in_dtype; qd.mag_exp = 22;
        const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
        int gave_up = 0;
        // chunk ch of a paired input -> v; false while a pair of it does not carry this launch's epoch yet
        auto load_pairs = [&](int ch, float v[16]) {
            const int j0 = ch * 16;
            asm volatile("" ::: "memory");                  // another workgroup writes this memory: load again on every call
            // (device-scope loads, all eight requested before any is looked at; beyond the array the buffer returns zeros)
            v4u pr[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) pr[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (j0 + 2 * q) * 8, 0, 16);
            unsigned int ok = 1u, any = 0u;                 // all pairs of the chunk carry the epoch / at least one does
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int j = j0 + 2 * q;
                const unsigned int e0 = pr[q][1], e1 = pr[q][3];
                ok &= (unsigned int)(j >= op.N) | (unsigned int)(e0 == epoch);
                ok &= (unsigned int)(j + 1 >= op.N) | (unsigned int)(e1 == epoch);
                any |= (unsigned int)(j < op.N) & (unsigned int)(e0 == epoch);
                const unsigned int b0 = j < op.N ? pr[q][0] : 0u, b1 = j + 1 < op.N ? pr[q][2] : 0u;
                v[2 * q] = __builtin_bit_cast(float, b0);
                v[2 * q + 1] = __builtin_bit_cast(float, b1);
            }
            return ok | (any << 1);
        };
        // the same, repeated until the whole wave has its chunks (or the time is up: gave_up)
        auto wait_pairs = [&](int ch, float v[16]) {
            unsigned int spins = 0;
            const int j_wave = (ch - lane) * 16;            // first element of this wave's share
            for (;;) {
                const unsigned int got = load_pairs(ch, v);
                if (__builtin_amdgcn_ballot_w64((got & 1u) == 0u) == 0) return;
                // Not all there yet.  If part of the wave's share is, the producing phase is under way:
                // the wave asks again at once.  If nothing is, the wave polls its first pair only (one
                // transaction per round, all lanes the same address) until that one carries this launch's
                // epoch, so that workgroups waiting far ahead of the running phase leave the memory system alone.
                bool stop = false;
                const bool some = __builtin_amdgcn_ballot_w64((got & 2u) != 0u) != 0;
                for (; !some;) {
                    typedef unsigned int v2u __attribute__((ext_vector_type(2)));
                    asm volatile("" ::: "memory");
                    const v2u pr = __builtin_amdgcn_raw_buffer_load_b64(rsrc, j_wave * 8, 0, 16);
                    if (j_wave >= op.N || pr.y == epoch) break;
                    ++spins;
                    // (the clock and the error word are looked at every 16th round, and on the first: a limit of zero gives up at once)
                    if ((spins & 15u) == 1u)
                        stop = __builtin_amdgcn_s_memrealtime() - t0 > spin_ticks ||
                               __hip_atomic_load(&state->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
                    if (stop) break;
                    __builtin_amdgcn_s_sleep(8);
                }
                if (stop || __builtin_amdgcn_s_memrealtime() - t0 > spin_ticks) {
                    gave_up = 1;
                    return;
                }
            }
        };
        // v *= the input scale of chunk ch (as the quantiser of the streaming path does: one fp32 product)
        auto scale_chunk = [&](int ch, float v[16]) {
            if (!op.in_scale) return;
            const int j0 = ch * 16;
            if (j0 + 16 <= op.N) {
                const gptr_v4u sp = (gptr_v4u)(op.in_scale + j0);
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const v4u u = sp[q];
                    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        v[8 * q + 2 * i] *= half_bits_to_float((uint16_t)(w[i] & 0xFFFFu));
                        v[8 * q + 2 * i + 1] *= half_bits_to_float((uint16_t)(w[i] >> 16));
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (j0 + i < op.N) v[i] *= half_bits_to_float(((gptr_u16)op.in_scale)[j0 + i]);
            }
        };
        auto max_of = [&](const float v[16], float& m, int& bad) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float a = fabsf(v[i]);
                if (!(a <= 3.0e38f)) bad = 1;
                m = fmaxf(m, a);
            }
        };
        // A thread owns chunks tid, tid + 512, ...; inputs of up to 32768 elements (four chunks per thread: every input
        // the executor accepts, kExecMaxSteps) stay in registers between the maximum and the rounding; the other
        // branch, which fetches a longer input twice, is kept for a narrower workgroup.
        const int n_c = (n_chunks + kExecThreads - 1) / kExecThreads;           // chunks per thread
        const bool held = n_c <= kExecHeld;
        if (op.in_ll == 2) __syncthreads();                 // the LDS array of this workgroup's previous task is complete
        float hv[kExecHeld][16];
        float m = 0.f;
        int bad = 0;
        // chunk ch of the input, scaled, wherever it comes from (c: which of the thread's chunks, for the prefetched scales)
        auto fetch = [&](int ch, int c, float v[16]) {
            if (op.in_ll == 0) {
                if (ch < n_chunks) load_chunk16(qd, 0, ch, true, v);
                else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) v[i] = 0.f;
                }
                return;
            }
            if (op.in_ll == 1) {
                wait_pairs(ch, v);                          // (a chunk past the end reads as zeros)
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = ch * 16 + i < op.N ? lds_t[ch * 16 + i] : 0.f;
            }
            if (c < kExecHeld && op.in_scale && ch * 16 + 16 <= op.N) {
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const uint32_t w[4] = {sraw[c][q].x, sraw[c][q].y, sraw[c][q].z, sraw[c][q].w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        v[8 * q + 2 * i] *= half_bits_to_float((uint16_t)(w[i] & 0xFFFFu));
                        v[8 * q + 2 * i + 1] *= half_bits_to_float((uint16_t)(w[i] >> 16));
                    }
                }
            } else {
                scale_chunk(ch, v);
            }
        };
        // (a wave none of whose lanes owns a chunk goes straight to the barrier)
        const bool wave_works = tid - lane < n_chunks;
        if (held) {
#pragma unroll
            for (int c = 0; c < kExecHeld; ++c) {
                if (c < n_c && tid - lane + c * kExecThreads < n_chunks) {
                    fetch(tid + c * kExecThreads, c, hv[c]);
                    max_of(hv[c], m, bad);
                }
            }
        } else {
            for (int c = 0; c < n_c && !gave_up; ++c) {
                fetch(tid + c * kExecThreads, kExecHeld, hv[0]);
                max_of(hv[0], m, bad);
            }
        }
        if (wave_works) {
            m = wave_reduce32(m, [](float a, float b) { return fmaxf(a, b); });
            bad = __builtin_amdgcn_ballot_w64(bad != 0) != 0;
            if (lane == 0) {                                // one LDS atomic per wave
                atomicMax(lds_max, __builtin_bit_cast(unsigned int, m));      // m >= 0: its bits order like the value
                if (bad) atomicOr(lds_bad, 1);
            }
            if (gave_up) *lds_abort = 1;
        }
        __syncthreads();
        if (*lds_abort) break;                              // the whole workgroup leaves (same LDS word for all)
        m = __builtin_bit_cast(float, *lds_max);
        bad = *lds_bad;
        int ex = 0;
        float step = 1.0f;
        if (m > 0.f && !bad) {
            (void)frexpf(m, &ex);
            int se = ex - 22;
            se = se < -126 ? -126 : se;
            step = ldexpf(1.0f, se);
        }
        const float inv_step = 1.0f / step;
        if (wave_works) {
            long long local_sum = 0;
            if (held) {
#pragma unroll
                for (int c = 0; c < kExecHeld; ++c) {
                    const int ch = tid + c * kExecThreads;
                    if (c < n_c && ch < n_chunks)
                        local_sum += quantize_chunk16(hv[c], inv_step, bad != 0, (uint4*)lds_bq + bq_piece(ch, 0));
                }
            } else {
                for (int c = 0; c < n_c; ++c) {
                    const int ch = tid + c * kExecThreads;
                    fetch(ch, kExecHeld, hv[0]);            // (pairs this thread has already seen valid)
                    if (ch < n_chunks) local_sum += quantize_chunk16(hv[0], inv_step, bad != 0, (uint4*)lds_bq + bq_piece(ch, 0));
                }
            }
            local_sum = wave_sum64(local_sum);
            if (lane == 0) atomicAdd(lds_sum, (unsigned long long)local_sum);  // |sum| < 2^39: exact, whatever the order
        }
        __syncthreads();
        const double tot = (double)(long long)*lds_sum;
        const double two_step = bad ? (double)__builtin_nanf("") : 2.0 * (double)step;
        const double neg_qs = -tot * (double)step;

        // ---- the task's row blocks, 8 / W at a time ----
        const int per = kExecWaves >> tk.wl;
        const int n_grp = (tk.n_rb + per - 1) / per;
        const uint32_t b_lane = (uint32_t)(bq_piece(g, n < 3 ? n : 0) * 16);     // unused columns re-read slice 0
        for (int grp = 0; grp < n_grp; ++grp) {
            // (the output scales of the first group came with the task's first tiles; a later group requests its own now)
            if (grp > 0) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int idx = tid + u * kExecThreads;
                    const int rb = tk.rb0 + grp * per + (idx >> 7);
                    if (op.out_scale && idx < per * kTileRows && rb < tk.rb0 + tk.n_rb)
                        ps[u] = ((gptr_u16)op.out_scale)[rb * kTileRows + (idx & 127)];
                }
            }
            const uint16_t ps_now[2] = {ps[0], ps[1]};
            v4i acc[1][8];
#pragma unroll
            for (int p = 0; p < 8; ++p) acc[0][p] = v4i{0, 0, 0, 0};
            const int last = cnt > 0 ? cnt - 1 : 0;
            const int w_steps = w_of;
#define NQ_ISSUE(k)                                                              \
    do {                                                                         \
        wbuf[k] = load_tile_words(a_base, a_off);                                \
        a_off += (uint32_t)(w_steps * 1024);                                     \
    } while (0)
#define NQ_LDSB(i) (*(const v4u*)(lds_bq + b_lane + (part + ((i) < last ? (i) : last) * w_steps) * (int)kBqStepBytes))
            v4u bop[2][1];
            bop[0][0] = NQ_LDSB(0);
            for (int i0 = 0; i0 < cnt; i0 += D) {
#pragma unroll
                for (int k = 0; k < D; ++k) {
                    if (i0 + k < cnt) {
                        bop[(k + 1) & 1][0] = NQ_LDSB(i0 + k + 1);
                        mac_tile<1>(acc, wbuf[k], bop[k & 1]);
                        if (i0 + k + D < cnt) NQ_ISSUE(k);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
#undef NQ_LDSB
#undef NQ_ISSUE
            // the ring is empty: the next group's first tiles go out before the epilogue
            const int w_cur = 1 << tk.wl;
            if (grp + 1 < n_grp) NQ_PRIME(tk, grp + 1);

            // ---- epilogue: raw sums -> LDS, added over the W waves of a row block, scaled, stored ----
            __syncthreads();
            if (tid == 0 && grp == 0) {                     // every thread has read them; the next task starts from zero
                *lds_sum = 0;
                *lds_max = 0;
                *lds_bad = 0;
            }                                // the regions (and, after the last group, the input) are free
            if (n < 3) {
                v4i* dst = (v4i*)(lds_epi + wave * kExecEpiInts + n * kTileRows) + g;
#pragma unroll
                for (int p = 0; p < 8; ++p) dst[4 * p] = p == 7 ? -acc[0][p] : acc[0][p];    // rows 16p + 4g .. +3; plane 7 holds -128 * sum
            }
            __syncthreads();
#pragma unroll 1
            for (int u = 0; u < 2; ++u) {
                const int idx = tid + u * kExecThreads;
                if (idx >= per * kTileRows) break;          // (whole waves: per * 128 is a multiple of 64)
                const int sub = idx >> 7, row = idx & 127;
                const int rb = tk.rb0 + grp * per + sub;
                const int grow = rb * kTileRows + row;
                if (idx < per * kTileRows && rb < tk.rb0 + tk.n_rb && grow < op.M) {
                    int h = 0, mm = 0, l = 0;
                    const int* q = lds_epi + sub * w_cur * kExecEpiInts + row;
                    // (the waves' sums requested together; a wave beyond the row block's W reads wave 0's region again and is not added)
#pragma unroll 1
                    for (int w0 = 0; w0 < w_cur; w0 += kExecWaves) {
#pragma unroll
                        for (int w = 0; w < kExecWaves; ++w) {
                            const int* qw = q + (w0 + w < w_cur ? w0 + w : 0) * kExecEpiInts;
                            const int a0 = qw[0], a1 = qw[kTileRows], a2 = qw[2 * kTileRows];
                            h += w0 + w < w_cur ? a0 : 0;
                            mm += w0 + w < w_cur ? a1 : 0;
                            l += w0 + w < w_cur ? a2 : 0;
                        }
                    }
                    const double raw = fma((double)h, 65536.0, fma((double)mm, 256.0, (double)l));
                    const double val = fma(raw, __builtin_ldexp(two_step, -(row >> 4)), neg_qs);    // exact
                    float f = (float)val;                   // (rounded, then scaled in fp32: as the streaming kernels do)
                    if (op.out_scale) f *= half_bits_to_float(u ? ps_now[1] : ps_now[0]);
                    if (op.out) store_out(op.out, op.out_dtype, (size_t)grow, f, op.out_scale != nullptr);
                    if (op.out_lds) lds_t[grow] = f;
                    if (op.out_ll) {
                        // what a reader of the stored output would see: the value after its rounding to the output type
                        if (op.out_dtype == NQ_BF16) f = bf16_bits_to_float(float_to_bf16_bits(f));
                        else if (op.out_dtype == NQ_F16) f = half_bits_to_float(float_to_f16_bits(f));
                        ll_store(op.out_ll + grow, f, epoch);
                    }
                }
            }
        }
        // The next task's first tiles and scales go out now, behind this task's stores and ahead of the wait
        // for that task's input.  (Not earlier: vector memory returns in order, so anything this task still
        // had to wait for -- a scale, a spilled register -- would have waited for those tiles as well.)
        if (more) {
            NQ_PRIME(nxt, 0);
            NQ_PREFETCH_SCALES(nxt);
        }
        ++ti;
        tk = nxt;
    }
#undef NQ_PRIME
#undef NQ_PREFETCH_SCALES

    // ---- leave: report a missed deadline; the last workgroup out advances the epoch ----
    __syncthreads();
    if (tid == 0 && state) {
        if (*lds_abort) __hip_atomic_store(&state->error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned int left = __hip_atomic_fetch_add(&state->done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (left + 1 == gridDim.x) {
            __hip_atomic_store(&state->done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned int e = epoch + 1;
            __hip_atomic_store(&state->epoch, e == 0 ? 1u : e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

__global__ void __launch_bounds__(kExecThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
exec_kernel(const ExecTask* __restrict__ tasks, const int* __restrict__ task_begin,
            ExecState* __restrict__ state, int bq_bytes, unsigned long long spin_ticks)
{
    exec_body(tasks, task_begin[blockIdx.x], task_begin[blockIdx.x + 1], state, bq_bytes, spin_ticks);
}

// One small layer, both stages, by ONE workgroup in one launch: t stays in LDS between the stages
// (the two-stage GEMV of Appendix E.2 with its intermediate in shared memory).  The two task records are
// kernel arguments.
struct ExecPair {
    ExecTask t[2];
};
__global__ void __launch_bounds__(kExecThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
exec_small_kernel(ExecPair pair, int bq_bytes)
{
    exec_body(pair.t, 0, 2, nullptr, bq_bytes, 0ull);
}

// ---------------------------------------------------------------------------------------------
// host: the task lists
// ---------------------------------------------------------------------------------------------
struct PlannedTask {
    int wg, phase, layer, stage, rb0, n_rb, W;
};

// Levels are run as 2 phases each (stage 1 of every layer of the level, then stage 2).  Inside a
// phase the row blocks are dealt to the workgroups in runs of 8 / W with the largest W (waves per row
// block) for which every run finds a workgroup of its own; consecutive phases start where the one
// before stopped, so a workgroup's next task usually lies several phases ahead and its first tiles
// are in registers long before its input exists.  Every workgroup's list is in phase order, which
// is what makes the grid deadlock-free: the earliest unfinished phase depends on finished ones only.
static void plan_tasks(const int64_t* d_out, const int64_t* d_in, const int64_t* r, const int* level_of, int n,
                       int n_wg, std::vector<PlannedTask>& out)
{
    out.clear();
    int start = 0;
    for (int i0 = 0; i0 < n;) {
        int i1 = i0;
        while (i1 < n && level_of[i1] == level_of[i0]) ++i1;
        for (int stage = 0; stage < 2; ++stage) {
            const int phase = 2 * level_of[i0] + stage;
            std::vector<int> nrb(i1 - i0);
            for (int i = i0; i < i1; ++i) nrb[i - i0] = (int)n_rowblocks(stage == 0 ? r[i] : d_out[i]);
            int W = kExecWaves;
            auto runs = [&](int w) {
                int u = 0;
                for (int v : nrb) u += (v + kExecWaves / w - 1) / (kExecWaves / w);
                return u;
            };
            while (W > 1 && runs(W) > n_wg) W /= 2;
            const int per = kExecWaves / W;
            const int total = runs(W);
            // runs per workgroup when even one wave per row block leaves more runs than workgroups
            const int each = (total + n_wg - 1) / n_wg;
            int run = 0;
            for (int i = i0; i < i1; ++i) {
                for (int rb = 0; rb < nrb[i - i0]; rb += per, ++run) {
                    const int wg = (start + run / each) % n_wg;
                    const int cnt = std::min(per, nrb[i - i0] - rb);
                    if (!out.empty() && out.back().wg == wg && out.back().phase == phase && out.back().layer == i &&
                        out.back().rb0 + out.back().n_rb == rb)
                        out.back().n_rb += cnt;                 // the same workgroup goes on with the same layer
                    else
                        out.push_back(PlannedTask{wg, phase, i, stage, rb, cnt, W});
                }
            }
            start = (start + (total + each - 1) / each) % n_wg;
        }
        i0 = i1;
    }
}

}  // namespace nq

using namespace nq;

struct nq_exec_s {
    int n, n_wg, device;
    std::vector<nq_handle> handles;
    void* alloc;                    // tasks | task_begin | state | pairs
    ExecTask* tasks;
    int* task_begin;
    ExecState* state;
    int bq_bytes;
    size_t lds_bytes;
    int n_tasks;
};

static int exec_fail(int code, const char* msg)
{
    set_error(msg);
    return code;
}

extern "C" int nq_exec_plan_tasks(const int64_t* d_out, const int64_t* d_in, const int64_t* r, const int* level_of, int n,
                                  int n_workgroups, int32_t* tasks_out, int capacity, int* n_tasks)
{
    if (!d_out || !d_in || !r || !level_of || !n_tasks) return exec_fail(NQ_E_NULL, "nq_exec_plan_tasks: NULL pointer");
    if (n < 1 || n_workgroups < 1) return exec_fail(NQ_E_INVALID_ARG, "nq_exec_plan_tasks: n and n_workgroups must be >= 1");
    for (int i = 0; i < n; ++i) {
        if (d_out[i] < 1 || d_in[i] < 1 || r[i] < 1) return exec_fail(NQ_E_SHAPE, "nq_exec_plan_tasks: dimensions must be >= 1");
        if (level_of[i] < 0 || (i > 0 && level_of[i] < level_of[i - 1]))
            return exec_fail(NQ_E_INVALID_ARG, "nq_exec_plan_tasks: levels must be >= 0 and listed in order");
    }
    std::vector<PlannedTask> t;
    plan_tasks(d_out, d_in, r, level_of, n, n_workgroups, t);
    *n_tasks = (int)t.size();
    if (tasks_out) {
        if ((int)t.size() > capacity) return exec_fail(NQ_E_INVALID_ARG, "nq_exec_plan_tasks: tasks_out too small");
        for (size_t k = 0; k < t.size(); ++k) {
            int32_t* o = tasks_out + 7 * k;
            o[0] = t[k].wg; o[1] = t[k].phase; o[2] = t[k].layer; o[3] = t[k].stage; o[4] = t[k].rb0; o[5] = t[k].n_rb; o[6] = t[k].W;
        }
    }
    return NQ_OK;
}

// ---------------------------------------------------------------------------------------------
// a lone small layer at batch 1: both stages in one launch by one workgroup (see exec_small_kernel)
// ---------------------------------------------------------------------------------------------
namespace nq {

// Off by default: measured on config 1 (1024 x 1024, r = 256, 66 KB of bits) one workgroup doing all ten row
// blocks of the two stages in turn takes 13.3 us per forward where the two launches that spread them over ten
// CUs take 10.2 us -- on this chip the latency of a stage is a wave's instruction stream, not the launch, and a
// lone workgroup serialises what the CUs do side by side.  The option "small_layer_kb" gives the packed size
// (both factors, KiB) up to which a lone layer at batch 1 takes this path.
constexpr int kSmallLayerKiB = 0;

bool small_layer_fits(nq_handle h, int batch)
{
    if (batch != 1 || opt_flag(OPT_NO_SMALL_LAYER)) return false;
    if (h->d_in > 16384 || h->r > 8192) return false;       // one chunk per thread; t in LDS
    const size_t tile_bytes = (tile_words(h->r, h->d_in) + tile_words(h->d_out, h->r)) * 4;
    return tile_bytes <= (size_t)opt_or(OPT_SMALL_LAYER_KB, kSmallLayerKiB) * 1024;
}

int launch_small_layer(nq_handle h, const DecodeWorkspace& w, const void* x, void* y, bool unscaled, hipStream_t s)
{
    static bool attr_set = false;
    ExecPair p{};
    // waves per row block: as many as leave every row block of the stage a place in ONE round (else one wave each, several rounds)
    auto wl_for = [](int64_t n_rb) {
        int W = kExecWaves;
        while (W > 1 && n_rb * W > kExecWaves) W /= 2;
        int wl = 0;
        while ((1 << wl) < W) ++wl;
        return wl;
    };
    ExecTask& a = p.t[0];
    a.tiles = h->vt_tiles; a.in = x; a.in_ll = 0; a.in_scale = h->s_in; a.out_scale = nullptr;
    a.out = w.t; a.out_ll = nullptr; a.out_lds = 1;
    a.M = (int)h->r; a.N = (int)h->d_in; a.n_steps = (int)n_steps(h->d_in); a.in_dtype = h->x_dtype; a.out_dtype = NQ_F32;
    a.rb0 = 0; a.n_rb = (int)n_rowblocks(h->r); a.wl = wl_for(a.n_rb);
    ExecTask& b = p.t[1];
    b.tiles = h->u_tiles; b.in = nullptr; b.in_ll = 2; b.in_scale = h->s_mid; b.out_scale = unscaled ? nullptr : h->s_out;
    b.out = y; b.out_ll = nullptr; b.out_lds = 0;
    b.M = (int)h->d_out; b.N = (int)h->r; b.n_steps = (int)n_steps(h->r); b.in_dtype = NQ_F32; b.out_dtype = h->y_dtype;
    b.rb0 = 0; b.n_rb = (int)n_rowblocks(h->d_out); b.wl = wl_for(b.n_rb);
    const int bq_bytes = (int)std::max(n_steps(h->d_in), n_steps(h->r)) * (int)kBqStepBytes;
    const size_t lds_bytes = (size_t)bq_bytes + (size_t)kExecWaves * kExecEpiInts * 4 + 32 + (size_t)round_up(h->r, 16) * 4;
    if (!attr_set) {
        NQ_HIP(hipFuncSetAttribute((const void*)exec_small_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set = true;
    }
    hipLaunchKernelGGL(exec_small_kernel, dim3(1), dim3(kExecThreads), lds_bytes, s, p, bq_bytes);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

}  // namespace nq

extern "C" int nq_exec_destroy(nq_exec e)
{
    if (!e) return NQ_OK;
    (void)hipDeviceSynchronize();
    if (e->alloc) (void)hipFree(e->alloc);
    delete e;
    return NQ_OK;
}

extern "C" int nq_exec_create(nq_exec* out, const nq_handle* hs, const void* const* xs, void* const* ys,
                              const int* level_of, int n)
{
    if (!out) return exec_fail(NQ_E_NULL, "nq_exec_create: out is NULL");
    *out = nullptr;
    if (!hs || !xs || !ys || !level_of) return exec_fail(NQ_E_NULL, "nq_exec_create: NULL array");
    if (n < 1) return exec_fail(NQ_E_INVALID_ARG, "nq_exec_create: n must be >= 1");
    std::vector<int> src(n, -1);
    std::vector<char> consumed(n, 0);
    for (int i = 0; i < n; ++i) {
        nq_handle h = hs[i];
        if (!h) return exec_fail(NQ_E_NULL, "nq_exec_create: NULL handle in list");
        if (h->flags & NQ_FLAG_DECODE_VALU) return exec_fail(NQ_E_UNSUPPORTED, "nq_exec_create: handle uses NQ_FLAG_DECODE_VALU");
        if (h->device != hs[0]->device) return exec_fail(NQ_E_INVALID_ARG, "nq_exec_create: handles live on different devices");
        if (n_steps(h->d_in) > kExecMaxSteps || n_steps(h->r) > kExecMaxSteps)
            return exec_fail(NQ_E_SHAPE, "nq_exec_create: d_in and r must be <= 32768");
        if (level_of[i] < 0 || (i > 0 && level_of[i] < level_of[i - 1]))
            return exec_fail(NQ_E_INVALID_ARG, "nq_exec_create: levels must be >= 0 and listed in order");
        if (!xs[i] || !ys[i]) return exec_fail(NQ_E_NULL, "nq_exec_create: x or y is NULL");
        if (((uintptr_t)xs[i] | (uintptr_t)ys[i]) & 15u) return exec_fail(NQ_E_ALIGN, "nq_exec_create: x and y must be 16-byte aligned");
        for (int j = 0; j < i; ++j)
            if (hs[j] == h) return exec_fail(NQ_E_INVALID_ARG, "nq_exec_create: a handle appears twice");
    }
    // data flow: an input is either outside memory, or exactly the output of a layer of an earlier level
    auto bytes_x = [&](int i) { return (size_t)hs[i]->d_in * (hs[i]->x_dtype == NQ_F32 ? 4 : 2); };
    auto bytes_y = [&](int i) { return (size_t)hs[i]->d_out * (hs[i]->y_dtype == NQ_F32 ? 4 : 2); };
    auto overlap = [](const void* a, size_t na, const void* b, size_t nb) {
        return (const char*)a < (const char*)b + nb && (const char*)b < (const char*)a + na;
    };
    for (int i = 0; i < n; ++i) {
        for (int j = 0; j < n; ++j) {
            if (j != i && overlap(ys[i], bytes_y(i), ys[j], bytes_y(j)))
                return exec_fail(NQ_E_INVALID_ARG, "nq_exec_create: two outputs overlap");
            if (!overlap(xs[i], bytes_x(i), ys[j], bytes_y(j))) continue;
            const bool same = xs[i] == ys[j] && hs[i]->d_in == hs[j]->d_out && hs[i]->x_dtype == hs[j]->y_dtype;
            if (!same || level_of[j] >= level_of[i])
                return exec_fail(NQ_E_INVALID_ARG,
                                 "nq_exec_create: an input may overlap an output only by BEING the output (same pointer, "
                                 "length and type) of a layer of an earlier level");
            src[i] = j;
            consumed[j] = 1;
        }
    }

    nq_exec e = new (std::nothrow) nq_exec_s();
    if (!e) return exec_fail(NQ_E_HIP, "nq_exec_create: out of host memory");
    e->n = n; e->device = hs[0]->device; e->alloc = nullptr;
    e->handles.assign(hs, hs + n);
    // up to two workgroups per CU, and only as many as can be resident together
    int per_cu = 0;
    std::vector<int64_t> d_out(n), d_in(n), r(n);
    int max_steps = 4;
    for (int i = 0; i < n; ++i) {
        d_out[i] = hs[i]->d_out; d_in[i] = hs[i]->d_in; r[i] = hs[i]->r;
        max_steps = std::max(max_steps, (int)std::max(n_steps(d_in[i]), n_steps(r[i])));
    }
    e->bq_bytes = max_steps * (int)kBqStepBytes;
    e->lds_bytes = (size_t)e->bq_bytes + (size_t)kExecWaves * kExecEpiInts * 4 + 32;
    hipError_t he = hipFuncSetAttribute((const void*)exec_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (he == hipSuccess)
        he = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)exec_kernel, kExecThreads, e->lds_bytes);
    if (he != hipSuccess) { delete e; return hip_fail(he, "occupancy query (executor)", __FILE__, __LINE__); }
    if (per_cu < 1) { delete e; return exec_fail(NQ_E_UNSUPPORTED, "nq_exec_create: the executor's workgroup does not fit a CU"); }
    e->n_wg = device_cu_count() * std::min(per_cu, 2);

    std::vector<PlannedTask> planned;
    plan_tasks(d_out.data(), d_in.data(), r.data(), level_of, n, e->n_wg, planned);
    // per workgroup, in phase order (plan_tasks emits phases in order: a stable sort by workgroup keeps it)
    std::stable_sort(planned.begin(), planned.end(), [](const PlannedTask& a, const PlannedTask& b) { return a.wg < b.wg; });
    std::vector<int> begin(e->n_wg + 1, 0);
    for (size_t k = 0; k < planned.size(); ++k) begin[planned[k].wg + 1] += 1;
    for (int w = 0; w < e->n_wg; ++w) begin[w + 1] += begin[w];
    e->n_tasks = (int)planned.size();

    auto al = [](size_t v) { return (v + 255) / 256 * 256; };
    const size_t tasks_b = al(sizeof(ExecTask) * planned.size()), begin_b = al(sizeof(int) * begin.size()),
                 state_b = al(sizeof(ExecState));
    size_t pairs = 0;
    std::vector<size_t> t_off(n), y_off(n);
    for (int i = 0; i < n; ++i) {
        t_off[i] = pairs; pairs += al((size_t)hs[i]->r * 8);
        y_off[i] = pairs; if (consumed[i]) pairs += al((size_t)hs[i]->d_out * 8);
    }
    const size_t total = tasks_b + begin_b + state_b + pairs;
    he = hipMalloc(&e->alloc, total);
    if (he != hipSuccess) { delete e; return hip_fail(he, "hipMalloc(executor)", __FILE__, __LINE__); }
    char* c = (char*)e->alloc;
    e->tasks = (ExecTask*)c; c += tasks_b;
    e->task_begin = (int*)c; c += begin_b;
    e->state = (ExecState*)c; c += state_b;
    char* pair_base = c;
    // the two stages of every layer
    std::vector<ExecTask> ops(2 * n);
    for (int i = 0; i < n; ++i) {
        nq_handle h = hs[i];
        ExecTask& a = ops[2 * i];
        a = ExecTask{};
        a.tiles = h->vt_tiles;
        a.in = src[i] >= 0 ? (const void*)(pair_base + y_off[src[i]]) : xs[i];
        a.in_ll = src[i] >= 0;
        a.in_scale = h->s_in; a.out_scale = nullptr;
        a.out = h->ws.t;                                   // (so that nq_binlr_read_intermediate sees it)
        a.out_ll = (unsigned long long*)(pair_base + t_off[i]);
        a.M = (int)h->r; a.N = (int)h->d_in; a.n_steps = (int)n_steps(h->d_in);
        a.in_dtype = h->x_dtype; a.out_dtype = NQ_F32;
        ExecTask& b = ops[2 * i + 1];
        b = ExecTask{};
        b.tiles = h->u_tiles;
        b.in = pair_base + t_off[i]; b.in_ll = 1;
        b.in_scale = h->s_mid; b.out_scale = h->s_out;
        b.out = ys[i];
        b.out_ll = consumed[i] ? (unsigned long long*)(pair_base + y_off[i]) : nullptr;
        b.M = (int)h->d_out; b.N = (int)h->r; b.n_steps = (int)n_steps(h->r);
        b.in_dtype = NQ_F32; b.out_dtype = h->y_dtype;
    }
    std::vector<ExecTask> tasks(planned.size());
    for (size_t k = 0; k < planned.size(); ++k) {
        tasks[k] = ops[2 * planned[k].layer + planned[k].stage];
        tasks[k].rb0 = planned[k].rb0;
        tasks[k].n_rb = planned[k].n_rb;
        int wl = 0;
        while ((1 << wl) < planned[k].W) ++wl;
        tasks[k].wl = wl;
    }
    ExecState st0{1u, 0u, 0, 0};
    he = hipMemset(e->alloc, 0, total);
    if (he == hipSuccess) he = hipMemcpy(e->tasks, tasks.data(), sizeof(ExecTask) * tasks.size(), hipMemcpyHostToDevice);
    if (he == hipSuccess) he = hipMemcpy(e->task_begin, begin.data(), sizeof(int) * begin.size(), hipMemcpyHostToDevice);
    if (he == hipSuccess) he = hipMemcpy(e->state, &st0, sizeof st0, hipMemcpyHostToDevice);
    if (he == hipSuccess) he = hipDeviceSynchronize();
    if (he != hipSuccess) {
        (void)hipFree(e->alloc);
        delete e;
        return hip_fail(he, "upload (executor)", __FILE__, __LINE__);
    }
    *out = e;
    return NQ_OK;
}

extern "C" int nq_exec_forward(nq_exec e, void* stream)
{
    if (!e) return exec_fail(NQ_E_NULL, "nq_exec_forward: NULL executor");
    // wall-clock limit of every wait, in ticks of the 100 MHz constant clock (default 2 s)
    const int us = opt(OPT_EXEC_SPIN_LIMIT_US);
    const unsigned long long ticks = us >= 0 ? (unsigned long long)us * 100ull : 200000000ull;
    hipLaunchKernelGGL(exec_kernel, dim3(e->n_wg), dim3(kExecThreads), e->lds_bytes, (hipStream_t)stream, e->tasks,
                       e->task_begin, e->state, e->bq_bytes, ticks);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

extern "C" int nq_exec_status(nq_exec e, void* stream)
{
    if (!e) return exec_fail(NQ_E_NULL, "nq_exec_status: NULL executor");
    NQ_HIP(hipStreamSynchronize((hipStream_t)stream));
    ExecState st;
    NQ_HIP(hipMemcpy(&st, e->state, sizeof st, hipMemcpyDeviceToHost));
    if (st.error) {
        // clear the word (and the count of a launch that may have been cut short cannot be off: every workgroup leaves through it)
        int zero = 0;
        NQ_HIP(hipMemcpy(&e->state->error, &zero, sizeof zero, hipMemcpyHostToDevice));
        return exec_fail(NQ_E_TIMEOUT, "nq_exec_status: a wait inside the executor ran into its time limit; outputs of that launch are incomplete");
    }
    return NQ_OK;
}

extern "C" int nq_exec_info(nq_exec e, int* n_workgroups, int* n_tasks, size_t* lds_bytes)
{
    if (!e) return exec_fail(NQ_E_NULL, "nq_exec_info: NULL executor");
    if (n_workgroups) *n_workgroups = e->n_wg;
    if (n_tasks) *n_tasks = e->n_tasks;
    if (lds_bytes) *lds_bytes = e->lds_bytes;
    return NQ_OK;
}
