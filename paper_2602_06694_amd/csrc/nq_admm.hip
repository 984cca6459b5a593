// Latent-binary ADMM on one matrix in binary64 (Section 3.2 Step 2-2 and 2-3; Appendix B): the dense
// products on the fp64 matrix cores, a blocked Cholesky with its inverse, the SVID proxy update by power
// iteration, the dual update and the magnitude balancing.  Host code only sequences launches.
#include "nq_internal.h"
#include "nq_lb_admm.h"

#include <math.h>
#include <algorithm>
#include <mutex>

namespace nq {

typedef double v4d __attribute__((ext_vector_type(4)));

// ============================================================================================
//  C = alpha op(A) op(B) + beta Cin + diag I   [, C2 = C + E]        (batched along blockIdx.z)
// ============================================================================================
struct GemmArgs {
    const double* A;
    const double* B;
    const double* Cin;     // read only when beta != 0 (may be C)
    double* C;
    const double* E;       // optional second output C2 = C + E (both with ldc)
    double* C2;
    int M, N, K;
    int lda, ldb, ldcin, ldc;
    long long sA, sB, sC;  // elements between batch members (Cin, C share sC)
    int trans_a;           // 0: A stored [M][K];  1: stored [K][M]
    int trans_b;           // 0: B stored [K][N];  1: stored [N][K]
    double alpha, beta, diag;
    int tile;              // 0: by size; 1 / 2 / 3: 128 x 128, 128 x 64, 64 x 64 (an in-place product needs a tile as wide as N)
    int lower_only;        // tiles that lie entirely above the diagonal are skipped
    int k_from_max;        // the reduction starts at max(first row, first column) of the tile: both operands
                           // are lower triangular in the sense  op(A)[i][k] = 0 for k < i,  op(B)[k][j] = 0 for k < j
    int k_parts;           // > 1 (unbatched only): blockIdx.z takes the reduction range [z, z + 1) * k_per_part and
    int k_per_part;        // writes its partial product to Cp[z]; beta, Cin and diag apply to part 0 only
    int lds_pad;           // bytes of LDS requested beyond the kernel's need (fewer workgroups per CU, room for other launches)
    int prio;              // the waves raise their priority: a launch on the critical path that shares the CUs with a
                           // long product on another stream then gets the issue slots first
    double* Cp[8];
};

constexpr int kGemmThreads = 256;
constexpr int kBK = 16;        // reduction depth of one LDS tile = four 16x16x4 matrix instructions

// A workgroup of four waves (2 x 2) owns a BM x BN tile of C; each wave (BM/2) x (BN/2) of it as
// 16 x 16 accumulator tiles.  v_mfma_f64_16x16x4_f64: lane l supplies A[l & 15][l >> 4] and B[l >> 4][l & 15],
// and holds C[4 v + (l >> 4)][l & 15] in element v of its four accumulators.  Operand tiles go through LDS, double
// buffered: the global loads of tile kt + 1 are in flight while tile kt is multiplied.  The LDS layout of an
// operand follows the memory layout of its source, so that both the staging stores and the operand reads are
// free of bank conflicts: a source that is contiguous along the reduction (A stored [M][K], B stored [N][K]) is kept
// as [i][k] with a row pitch of 17 doubles, one that is contiguous along the tile's rows or columns as [k][i] with
// a pitch of BM + 16.  Two workgroups fit a CU (registers and LDS), so one's staging overlaps the other's products.
// PF: tiles held in registers ahead of the one being multiplied (1 for the large tiles; 4 for the 64 x 64 tile, whose
// launches are mostly short reductions that would otherwise wait a full memory latency per 16 columns).
// TA, TB: the transpose flags as compile-time constants (LDS offsets become immediates of the LDS instructions).
template <int BM, int BN, int PF, bool TA, bool TB>
__device__ __forceinline__ void dgemm_body(const GemmArgs& g, const int bx, const int by, const int bz, double* lds_gemm)
{
    constexpr int PK = kBK + 1;
    constexpr int PA = BM + 16, PB = BN + 16;
    constexpr int SA = BM * PK > kBK * PA ? BM * PK : kBK * PA;
    constexpr int SB = BN * PK > kBK * PB ? BN * PK : kBK * PB;
    constexpr int TM = BM / 32, TN = BN / 32;
    constexpr int LA = BM * kBK / kGemmThreads, LB = BN * kBK / kGemmThreads;
    double* As = lds_gemm;                 // [2][SA]
    double* Bs = lds_gemm + 2 * SA;        // [2][SB]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i0 = by * BM, j0 = bx * BN;
    if (g.lower_only && j0 > i0 + BM - 1) return;
    if (g.prio) __builtin_amdgcn_s_setprio(2);
    const double* A = g.A + (size_t)(g.k_parts > 1 ? 0 : bz) * g.sA;
    const double* B = g.B + (size_t)(g.k_parts > 1 ? 0 : bz) * g.sB;
    const int part = g.k_parts > 1 ? bz : 0;
    const int zb = g.k_parts > 1 ? 0 : bz;
    const int k_begin = g.k_from_max ? ((i0 > j0 ? i0 : j0) / kBK) * kBK : part * g.k_per_part;
    const int k_end = g.k_parts > 1 && k_begin + g.k_per_part < g.K ? k_begin + g.k_per_part : g.K;
    const int n_kt = k_end > k_begin ? (k_end - k_begin + kBK - 1) / kBK : 0;
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);
    constexpr bool ta = TA, tb = TB;
    // a tile that lies inside the matrix needs no masking of rows or columns
    const bool interior = i0 + BM <= g.M && j0 + BN <= g.N;

    // What a thread fetches does not change from tile to tile except for the reduction offset: the pointers (rows and
    // columns beyond the matrix are clamped to its last one and their values replaced by zero), the element's depth
    // inside a tile and its place in LDS are set up once; the loop only advances the pointers.  Tiles are fetched in
    // ascending order, one call per tile.
    double ra[PF][LA], rb[PF][LB];
    const double* pa[LA];
    const double* pb[LB];
    bool va[LA], vb[LB];
    int ka[LA], kb[LB], sa[LA], sb[LB];
    const size_t step_a = ta ? (size_t)kBK * g.lda : kBK, step_b = tb ? kBK : (size_t)kBK * g.ldb;
#pragma unroll
    for (int p = 0; p < LA; ++p) {
        const int idx = p * kGemmThreads + tid;
        const int i = ta ? idx % BM : idx / kBK, k = ta ? idx / BM : idx % kBK;
        const int gi = i0 + i < g.M ? i0 + i : g.M - 1;
        va[p] = i0 + i < g.M;
        ka[p] = k;
        sa[p] = ta ? k * PA + i : i * PK + k;
        pa[p] = ta ? A + (size_t)(k_begin + k) * g.lda + gi : A + (size_t)gi * g.lda + k_begin + k;
    }
#pragma unroll
    for (int p = 0; p < LB; ++p) {
        const int idx = p * kGemmThreads + tid;
        const int j = tb ? idx / kBK : idx % BN, k = tb ? idx % kBK : idx / BN;
        const int gj = j0 + j < g.N ? j0 + j : g.N - 1;
        vb[p] = j0 + j < g.N;
        kb[p] = k;
        sb[p] = tb ? j * PK + k : k * PB + j;
        pb[p] = tb ? B + (size_t)gj * g.ldb + k_begin + k : B + (size_t)(k_begin + k) * g.ldb + gj;
    }
    auto fetch = [&](int kt, double (&ra)[LA], double (&rb)[LB]) {
        const int krem = k_end - (k_begin + kt * kBK);        // depth left, >= 1
        if (krem >= kBK && interior) {
#pragma unroll
            for (int p = 0; p < LA; ++p) ra[p] = *pa[p];
#pragma unroll
            for (int p = 0; p < LB; ++p) rb[p] = *pb[p];
        } else if (krem >= kBK) {                             // a whole tile: every address is inside the matrix
#pragma unroll
            for (int p = 0; p < LA; ++p) {
                const double v = *pa[p];
                ra[p] = va[p] ? v : 0.0;
            }
#pragma unroll
            for (int p = 0; p < LB; ++p) {
                const double v = *pb[p];
                rb[p] = vb[p] ? v : 0.0;
            }
        } else {                                              // the ragged last tile
#pragma unroll
            for (int p = 0; p < LA; ++p) ra[p] = (va[p] && ka[p] < krem) ? *pa[p] : 0.0;
#pragma unroll
            for (int p = 0; p < LB; ++p) rb[p] = (vb[p] && kb[p] < krem) ? *pb[p] : 0.0;
        }
#pragma unroll
        for (int p = 0; p < LA; ++p) pa[p] += step_a;
#pragma unroll
        for (int p = 0; p < LB; ++p) pb[p] += step_b;
    };
    auto stash = [&](int buf, const double (&ra)[LA], const double (&rb)[LB]) {
#pragma unroll
        for (int p = 0; p < LA; ++p) As[buf * SA + sa[p]] = ra[p];
#pragma unroll
        for (int p = 0; p < LB; ++p) Bs[buf * SB + sb[p]] = rb[p];
    };

    v4d acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = v4d{0.0, 0.0, 0.0, 0.0};

    // per-lane offsets of the operand reads: element (row l & 15 of a 16-row group, depth l >> 4 of a group of four)
    const int a_off = ta ? (lane >> 4) * PA + wm0 + (lane & 15) : (wm0 + (lane & 15)) * PK + (lane >> 4);
    constexpr int a_dk = ta ? 4 * PA : 4, a_dt = ta ? 16 : 16 * PK;
    const int b_off = tb ? (wn0 + (lane & 15)) * PK + (lane >> 4) : (lane >> 4) * PB + wn0 + (lane & 15);
    constexpr int b_dk = tb ? 4 : 4 * PB, b_dt = tb ? 16 * PK : 16;

#pragma unroll
    for (int t = 0; t < PF; ++t)
        if (t < n_kt) fetch(t, ra[t], rb[t]);
    if (n_kt > 0) stash(0, ra[0], rb[0]);
    __syncthreads();
    for (int kt0 = 0; kt0 < n_kt; kt0 += PF) {
#pragma unroll
        for (int sl = 0; sl < PF; ++sl) {
            const int kt = kt0 + sl;
            if (kt < n_kt) {
                const int buf = kt & 1;
                // slot sl went to LDS one tile ago: refill it with the tile PF ahead, multiply tile kt, then stage tile kt + 1
                if (kt + PF < n_kt) fetch(kt + PF, ra[sl], rb[sl]);
                const double* Ab = As + buf * SA + a_off;
                const double* Bb = Bs + buf * SB + b_off;
#pragma unroll
                for (int k4 = 0; k4 < kBK / 4; ++k4) {
                    double a[TM], b[TN];
#pragma unroll
                    for (int t = 0; t < TM; ++t) a[t] = Ab[k4 * a_dk + t * a_dt];
#pragma unroll
                    for (int t = 0; t < TN; ++t) b[t] = Bb[k4 * b_dk + t * b_dt];
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn)
                            acc[tm][tn] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
                }
                if (kt + 1 < n_kt) stash(buf ^ 1, ra[(sl + 1) % PF], rb[(sl + 1) % PF]);
                __syncthreads();
            }
        }
    }

    const bool first = part == 0;
    const double* Cin = g.Cin && first ? g.Cin + (size_t)zb * g.sC : nullptr;
    double* C = g.k_parts > 1 ? g.Cp[part] : g.C + (size_t)zb * g.sC;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = i0 + wm0 + tm * 16 + 4 * v + (lane >> 4);
                const int j = j0 + wn0 + tn * 16 + (lane & 15);
                if (i < g.M && j < g.N) {
                    double val = g.alpha * acc[tm][tn][v];
                    if (g.beta != 0.0 && first) val = fma(g.beta, Cin[(size_t)i * g.ldcin + j], val);
                    if (i == j && first) val += g.diag;
                    C[(size_t)i * g.ldc + j] = val;
                    if (g.C2) g.C2[(size_t)i * g.ldc + j] = val + g.E[(size_t)i * g.ldc + j];
                }
            }
}

template <int BM, int BN, int PF, bool TA, bool TB>
__global__ __launch_bounds__(kGemmThreads, 2) void dgemm_kernel(GemmArgs g)
{
    extern __shared__ __align__(16) double lds_dyn[];
    dgemm_body<BM, BN, PF, TA, TB>(g, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, lds_dyn);
}

template <int BM, int BN> constexpr size_t gemm_lds_bytes()
{
    constexpr int PK = kBK + 1;
    constexpr int SA = BM * PK > kBK * (BM + 16) ? BM * PK : kBK * (BM + 16);
    constexpr int SB = BN * PK > kBK * (BN + 16) ? BN * PK : kBK * (BN + 16);
    return (size_t)2 * (SA + SB) * sizeof(double);
}

constexpr int kGemmMaxLdsPad = 32768;

template <int BM, int BN, int PF, bool TA, bool TB> static int launch_gemm_variant(const GemmArgs& g, int batch, hipStream_t s)
{
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    constexpr size_t lds = gemm_lds_bytes<BM, BN>();
    std::call_once(once, [] {
        if (lds + kGemmMaxLdsPad > 65536)
            attr_err = hipFuncSetAttribute((const void*)dgemm_kernel<BM, BN, PF, TA, TB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)(lds + kGemmMaxLdsPad));
    });
    NQ_HIP(attr_err);
    dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM, batch);
    const size_t pad = (size_t)(g.lds_pad < 0 ? 0 : g.lds_pad > kGemmMaxLdsPad ? kGemmMaxLdsPad : g.lds_pad);
    hipLaunchKernelGGL((dgemm_kernel<BM, BN, PF, TA, TB>), grid, dim3(kGemmThreads), lds + pad, s, g);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

template <int BM, int BN, int PF> static int launch_gemm_tile(const GemmArgs& g, int batch, hipStream_t s)
{
    if (g.trans_a) return g.trans_b ? launch_gemm_variant<BM, BN, PF, true, true>(g, batch, s) : launch_gemm_variant<BM, BN, PF, true, false>(g, batch, s);
    return g.trans_b ? launch_gemm_variant<BM, BN, PF, false, true>(g, batch, s) : launch_gemm_variant<BM, BN, PF, false, false>(g, batch, s);
}

// Tile choice: the largest tile that still gives every CU two workgroups; the option "dgemm_tile" (1: 128 x 128,
// 2: 128 x 64, 3: 64 x 64) overrides it.
static int launch_gemm(const GemmArgs& g, int batch, hipStream_t s)
{
    if (g.M < 1 || g.N < 1 || batch < 1) return NQ_OK;
    auto tiles = [&](int bm, int bn) {            // workgroups that do work (with lower_only: those not entirely above the diagonal)
        const int tr = (g.M + bm - 1) / bm, tc = (g.N + bn - 1) / bn;
        long long n = 0;
        for (int i = 0; i < tr; ++i) n += g.lower_only ? std::min(tc, (i * bm + bm - 1) / bn + 1) : tc;
        return n * batch;
    };
    int choice = g.tile ? g.tile : opt_or(OPT_DGEMM_TILE, 0);
    if (choice < 1 || choice > 3) choice = tiles(128, 128) >= 512 ? 1 : tiles(128, 64) >= 384 ? 2 : 3;
    if (choice == 1) return launch_gemm_tile<128, 128, 1>(g, batch, s);
    if (choice == 2) return launch_gemm_tile<128, 64, 1>(g, batch, s);
    return launch_gemm_tile<64, 64, 4>(g, batch, s);
}

__host__ __device__ static GemmArgs gemm_args(int ta, int tb, int M, int N, int K, double alpha, const double* A, int lda, const double* B, int ldb,
                          double beta, const double* Cin, int ldcin, double* C, int ldc)
{
    GemmArgs g{};
    g.A = A; g.B = B; g.Cin = Cin; g.C = C; g.E = nullptr; g.C2 = nullptr;
    g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldcin = ldcin; g.ldc = ldc;
    g.sA = g.sB = g.sC = 0;
    g.trans_a = ta; g.trans_b = tb; g.alpha = alpha; g.beta = beta; g.diag = 0.0;
    g.tile = 0; g.lower_only = 0; g.k_from_max = 0;
    g.k_parts = 1; g.k_per_part = 0; g.prio = 0; g.lds_pad = 0;
    for (double*& c : g.Cp) c = nullptr;
    return g;
}

// ============================================================================================
//  Cholesky of one diagonal block and the inverse of its factor (one workgroup)
// ============================================================================================
constexpr int kNB = 64;        // width of a block column of the factorisation (an earlier 128-wide diagonal-block kernel measured slower than two of 64)

__device__ __forceinline__ double readlane_f64(double v, int lane)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
    return __hiloint2double(hi, lo);
}

// NB x NB block (NB = 64; every panel has an LDS buffer of its own, which a 128-wide block would not fit), (NB/4)^2 threads; a thread keeps one 4 x 4 sub-block of the matrix (a) and of the running
// right-hand side of L X = I (b, starts as the identity) in registers: row group ty = lane mod NB/4, column group tx.
// The column groups are dealt to the waves in turn (tx = wave + waves x (lane / (NB/4))), so that consecutive panels of
// four columns belong to different waves, and the elimination is a pipeline over panels without workgroup barriers:
//   * the wave that owns panel j + 1 applies panel j to that panel's columns only, factorises it on its own -- pivot and
//     multipliers travel by lane reads, the square root and its reciprocal come from the hardware's reciprocal-square-root
//     estimate refined by two coupled Newton steps and a residual correction (ten dependent operations; within an ulp
//     or two) -- publishes the four scaled columns (zero at and above their pivot) and the reciprocal pivots in the
//     panel's own LDS buffer, and raises the count of published panels;
//   * every wave, for each panel in order: waits until it is published, lets the threads that hold rows of the panel
//     finish those rows of X with the panel's 4 x 4 triangle and hand them to their column group by lane shuffles, and
//     applies the rank-4 update to its blocks right of the panel (a) and below it (b).
// So the chain of dependent operations per panel is "four columns of one wave" (about 2300 cycles), not that plus a whole
// rank-4 update and a barrier (4700): the other waves' updates run beside the next panel's factorisation.
// A wave waits only for panels with a smaller number than any it still has to publish, so the waits end; they also give
// up after a fixed number of polls (status is then set and the results are meaningless, every thread still finishes).
// H (lower part) is overwritten by L; the block of Linv receives L^-1 with an exactly zero upper part.  A pivot that is
// not > 0 sets *status (the results are then meaningless, every thread still finishes).
// pre != nullptr: first  A <- A - P P^T  with P = pre [NB][NB] (leading dimension ldh): the block's own tile of the
// trailing update of the block column before it, so that the update's other tiles can run beside this kernel's work.
// lds: potrf_lds_bytes<NB>() bytes.
template <int NB> constexpr size_t potrf_lds_bytes() { return (size_t)((NB / 4) * 4 * NB + (NB / 4) * 4) * sizeof(double) + 16; }

template <int NB>
__device__ __forceinline__ void potrf_inv_body(double* H, int ldh, double* Linv, int ldi, int o, int* status, int prio, const double* pre,
                                               double* lds)
{
    if (prio) __builtin_amdgcn_s_setprio(3);
    static_assert(NB == 64, "one LDS buffer per panel: 32 KiB at NB = 64");
    constexpr int G = NB / 4;                      // row groups of a column group = lanes they occupy; also the number of panels
    constexpr int CGW = 64 / G;                    // column groups per wave
    constexpr int NW = G / CGW;                    // waves
    double (*const colL)[4][NB] = (double (*)[4][NB])lds;
    double (*const dinv)[4] = (double (*)[4])(lds + G * 4 * NB);
    int& published = *(int*)(lds + G * 4 * NB + G * 4);            // panels whose columns are in LDS
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int local = lane / G;                    // which of the wave's column groups
    const int tx = wave + NW * local, ty = lane % G;
    double a[4][4], b[4][4];
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            a[ii][cc] = H[(size_t)(o + 4 * ty + ii) * ldh + o + 4 * tx + cc];
            b[ii][cc] = (4 * ty + ii == 4 * tx + cc) ? 1.0 : 0.0;
        }
    if (pre) {
        // P transposed into LDS (where the panels will go): thread t brings 16 entries of row t mod NB
        static_assert(NB * NB <= G * 4 * NB, "P fits the panel buffers");
        double* const pT = lds;                    // [NB][NB]: pT[k][row]
        {
            const int row = threadIdx.x % NB, k0 = (threadIdx.x / NB) * (NB * NB / (G * G));
            const double* src = pre + (size_t)row * ldh + k0;
#pragma unroll
            for (int k = 0; k < NB * NB / (G * G); ++k) pT[(k0 + k) * NB + row] = src[k];
        }
        __syncthreads();
#pragma unroll 4
        for (int k = 0; k < NB; ++k) {
            double pr[4], pc[4];
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) pr[ii] = pT[k * NB + 4 * ty + ii];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) pc[cc] = pT[k * NB + 4 * tx + cc];
#pragma unroll
            for (int ii = 0; ii < 4; ++ii)
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) a[ii][cc] = fma(-pr[ii], pc[cc], a[ii][cc]);
        }
        __syncthreads();                           // everybody has read P: the buffers change hands
    }
    if (threadIdx.x == 0) published = 0;
    __syncthreads();
    bool bad = false;

    // factorises panel jb (called by every lane of the wave that owns it) and publishes it
    auto factor_panel = [&](int jb) {
        const int src = G * (jb / NW) + jb;                // lane of the thread that holds the panel's diagonal block
        const bool mine = tx == jb;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int j = 4 * jb + jj;
            const double piv = readlane_f64(a[jj][jj], src);
            if (!(piv > 0.0)) bad = true;
            const double y = __builtin_amdgcn_rsq(piv);
            double g = piv * y, h = 0.5 * y;
            double e = fma(-h, g, 0.5);
            g = fma(g, e, g);
            h = fma(h, e, h);
            e = fma(-h, g, 0.5);
            g = fma(g, e, g);
            h = fma(h, e, h);
            e = fma(-g, g, piv);
            g = fma(e, h, g);
            const double d = g, inv = 2.0 * h;
            double l[4];
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                const int row = 4 * ty + ii;
                l[ii] = row > j ? a[ii][jj] * inv : 0.0;
                if (mine && row >= j) a[ii][jj] = row == j ? d : l[ii];
            }
#pragma unroll
            for (int cc = jj + 1; cc < 4; ++cc) {
                const double lc = readlane_f64(a[cc][jj], src);       // L[4 jb + cc][j]
                if (mine)
#pragma unroll
                    for (int ii = 0; ii < 4; ++ii) a[ii][cc] = fma(-l[ii], lc, a[ii][cc]);
            }
            if (mine)
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) colL[jb][jj][4 * ty + ii] = l[ii];
            if (lane == src) dinv[jb][jj] = inv;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");         // the columns are in LDS before the count says so
        if (lane == 0) __hip_atomic_store(&published, jb + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };

    if (wave == 0) factor_panel(0);
    for (int jb = 0; jb < G; ++jb) {
        // wait for panel jb (its owner published it one round ago, or just now)
        for (int spins = 0; __hip_atomic_load(&published, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) <= jb; ++spins) {
            if (spins > (1 << 22)) {
                bad = true;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        // the next panel's owner brings that panel's columns up to date first, factorises and publishes them
        if (jb + 1 < G && wave == (jb + 1) % NW) {
            if (tx == jb + 1) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) {
                        const double lc = colL[jb][q][4 * tx + cc];
#pragma unroll
                        for (int ii = 0; ii < 4; ++ii) a[ii][cc] = fma(-colL[jb][q][4 * ty + ii], lc, a[ii][cc]);
                    }
                }
            }
            factor_panel(jb + 1);
        }
        if (ty == jb) {                                    // rows 4 jb .. 4 jb + 3 of X
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    double acc = b[q][cc];
#pragma unroll
                    for (int p = 0; p < q; ++p) acc = fma(-colL[jb][p][4 * jb + q], b[p][cc], acc);
                    b[q][cc] = acc * dinv[jb][q];
                }
        }
        // the rank-4 update: everything it reads is requested first (LDS reads and lane shuffles have a long latency and
        // there is one wave per SIMD to hide it), then the 128 multiply-adds
        double lr[4][4], lc[4][4], xs[4][4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) lr[q][ii] = colL[jb][q][4 * ty + ii];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) lc[q][cc] = colL[jb][q][4 * tx + cc];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) xs[q][cc] = __shfl(b[q][cc], (lane & (64 - G)) | jb);
        }
        if (tx > jb + 1) {                                 // (column group jb + 1 was brought up to date above)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int cc = 0; cc < 4; ++cc)
#pragma unroll
                    for (int ii = 0; ii < 4; ++ii) a[ii][cc] = fma(-lr[q][ii], lc[q][cc], a[ii][cc]);
        }
        if (ty > jb) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int ii = 0; ii < 4; ++ii)
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) b[ii][cc] = fma(-lr[q][ii], xs[q][cc], b[ii][cc]);
        }
    }
#pragma unroll
    for (int ii = 0; ii < 4; ++ii)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const int i = 4 * ty + ii, c = 4 * tx + cc;
            if (c <= i) H[(size_t)(o + i) * ldh + o + c] = a[ii][cc];
            Linv[(size_t)(o + i) * ldi + o + c] = (c <= i) ? b[ii][cc] : 0.0;
        }
    if (bad) *status = 1;
}

template <int NB>
__global__ __launch_bounds__((NB / 4) * (NB / 4)) void potrf_inv_kernel(double* H, int ldh, double* Linv, int ldi, int o, int* status, int prio)
{
    extern __shared__ __align__(16) double lds_dyn[];
    potrf_inv_body<NB>(H, ldh, Linv, ldi, o, status, prio, nullptr, lds_dyn);
}

// One launch per block column k of the factorisation, after the diagonal block k has been factorised and inverted
// (X = L11^-1): the panel  P = A21 X^T  (the rows of L below the diagonal block), the trailing update  A22 -= P P^T
// (lower tiles), and the factorisation of the next diagonal block.  Nothing is handed from one workgroup to another:
//   * workgroup (0, 0) forms the first 64 rows of P, stores them as that block of L, applies  P P^T  to the diagonal
//     block k + 1 in its registers and factorises it (the long pole of the launch);
//   * workgroup (j, i + 1), j <= i, (i, j) != (0, 0), owns tile (i, j) of the trailing matrix: it forms the rows P_i and
//     P_j of the panel for itself (three 64 x 64 x 64 products instead of one; they cost little next to the
//     factorisation beside them), keeps them in its own piece of a scratch matrix -- or, tile (i, 0), stores P_i as
//     block i of L -- and subtracts  P_i P_j^T  from its tile.
// The panel is NOT written over A21: other workgroups still read A21, so L's blocks below the diagonal go to a matrix
// of their own (Lb; the diagonal blocks of L stay in H).  A step is then one launch of the factorisation's length
// where the panel, the update and the factorisation as launches of their own take three.
struct StepArgs {
    double* H;          // [..][ld]: A21, A22 (read and updated in place), diagonal blocks of L
    double* Lb;         // [..][ld]: L below the diagonal
    double* Linv;       // [..][ld]: the inverted diagonal blocks
    double* scratch;    // tiles (tiles + 1) / 2 pieces of 2 x 64 x 64
    int ld, o, prio;    // o: first row / column of block column k
    int* status;
};

__global__ __launch_bounds__(kGemmThreads, 2) void chol_step_kernel(StepArgs a)
{
    static_assert(kGemmThreads == (kNB / 4) * (kNB / 4) && kNB == 64, "both bodies are written for 256 threads and 64-wide blocks");
    extern __shared__ __align__(16) double lds_dyn[];
    const int ld = a.ld;
    const double* const X = a.Linv + (size_t)a.o * ld + a.o;
    double* const A21 = a.H + (size_t)(a.o + kNB) * ld + a.o;
    double* const L21 = a.Lb + (size_t)(a.o + kNB) * ld + a.o;
    if (blockIdx.y == 0) {
        if (blockIdx.x != 0) return;
        GemmArgs g = gemm_args(0, 1, kNB, kNB, kNB, 1.0, A21, ld, X, ld, 0.0, nullptr, 0, L21, ld);
        g.prio = a.prio;
        dgemm_body<64, 64, 4, false, true>(g, 0, 0, 0, lds_dyn);
        __syncthreads();                           // P's first rows are in memory (and LDS is free again)
        potrf_inv_body<kNB>(a.H, ld, a.Linv, ld, a.o + kNB, a.status, a.prio, L21, lds_dyn);
        return;
    }
    const int i = (int)blockIdx.y - 1, j = (int)blockIdx.x;
    if (j > i || i == 0) return;                   // above the diagonal; (0, 0) is the diagonal block's
    double* const mine = a.scratch + (size_t)(i * (i + 1) / 2 + j) * (2 * kNB * kNB);
    double* const Pi = j == 0 ? L21 + (size_t)i * kNB * ld : mine;
    const int ldi = j == 0 ? ld : kNB;
    double* const Pj = j == i ? Pi : mine + kNB * kNB;
    const int ldj = j == i ? ldi : kNB;
    GemmArgs g = gemm_args(0, 1, kNB, kNB, kNB, 1.0, A21 + (size_t)i * kNB * ld, ld, X, ld, 0.0, nullptr, 0, Pi, ldi);
    g.prio = a.prio;
    dgemm_body<64, 64, 4, false, true>(g, 0, 0, 0, lds_dyn);
    if (j != i) {
        g = gemm_args(0, 1, kNB, kNB, kNB, 1.0, A21 + (size_t)j * kNB * ld, ld, X, ld, 0.0, nullptr, 0, Pj, kNB);
        dgemm_body<64, 64, 4, false, true>(g, 0, 0, 0, lds_dyn);
    }
    __syncthreads();                               // this workgroup's P_i, P_j are in memory
    double* const Cij = a.H + (size_t)(a.o + kNB + i * kNB) * ld + a.o + kNB + j * kNB;
    g = gemm_args(0, 1, kNB, kNB, kNB, -1.0, Pi, ldi, Pj, ldj, 1.0, Cij, ld, Cij, ld);
    dgemm_body<64, 64, 4, false, true>(g, 0, 0, 0, lds_dyn);
}

// A += B, both [rows][cols] without padding (the two halves of a product whose reduction was split).
__global__ void add_half_kernel(double* A, const double* B, size_t count)
{
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += (size_t)gridDim.x * blockDim.x) A[e] += B[e];
}

// A += the other parts, in their order, on the leading r x r part of [rp][rp] matrices (the partial Gram products of a
// split reduction; part 0 is A itself).
struct GramParts {
    const double* p[8];
    int n;
};
__global__ void add_parts_kernel(double* A, GramParts parts, int rp, int r)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= r) return;
    const size_t at = (size_t)blockIdx.y * rp + j;
    double v = A[at];
    for (int q = 1; q < parts.n; ++q) v += parts.p[q][at];
    A[at] = v;
}

// Identity outside the leading r x r part of a [rp][rp] matrix (the padding that keeps the block algorithms
// exact: an identity block factorises and inverts to itself); `zero_inside` also clears the leading part.
__global__ void pad_identity_kernel(double* A, int rp, int r, int zero_inside)
{
    const size_t n = (size_t)rp * rp;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (size_t)gridDim.x * blockDim.x) {
        const int i = (int)(e / rp), j = (int)(e % rp);
        if (i >= r || j >= r) A[e] = (i == j) ? 1.0 : 0.0;
        else if (zero_inside) A[e] = 0.0;
    }
}

// ============================================================================================
//  SVID: power iteration on |P| and the proxy / dual update
// ============================================================================================
constexpr int kRowsPerWg = 16;

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// Sum over the workgroup of one value per thread (256 threads); every thread gets the result.
__device__ __forceinline__ double block_sum(double v, double* scratch4)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch4[threadIdx.x >> 6] = v;
    __syncthreads();
    return (scratch4[0] + scratch4[1]) + (scratch4[2] + scratch4[3]);
}

constexpr int kWParts = 8;      // the vector of a round is kept as eight partial vectors, added in a fixed order by its readers

__device__ __forceinline__ double w_at(const double* w8, int r, int k)
{
    return ((w8[k] + w8[r + k]) + (w8[2 * r + k] + w8[3 * r + k])) + ((w8[4 * r + k] + w8[5 * r + k]) + (w8[6 * r + k] + w8[7 * r + k]));
}

// One round of the power iteration in one pass over P [n][r]: for the 16 rows of this workgroup
//     a_i = sum_k |P[i][k]| b_k          with b = w / ||w||   (w: the unnormalised vector of the round before)
// and, unless `rows_only`, this workgroup's part of the next unnormalised vector  w'_k = sum_i |P[i][k]| a_i
// (partial[g][k]; a second kernel adds the parts in a fixed order).  `ones`: a_i = 1 instead (the start vector;
// its scale does not matter, the next round normalises).  w is staged in LDS (dynamic, r doubles).
__global__ __launch_bounds__(256) void power_pass_kernel(const double* P, int n, int r, const double* w8, int ones, int rows_only,
                                                          double* a_out, double* partial)
{
    extern __shared__ __align__(16) double w_s[];
    __shared__ double red[4];
    __shared__ double a_s[kRowsPerWg];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row0 = blockIdx.x * kRowsPerWg;
    if (!ones) {
        double q = 0.0;
        for (int k = tid; k < r; k += 256) {
            const double v = w_at(w8, r, k);
            w_s[k] = v;
            q = fma(v, v, q);
        }
        const double inv = 1.0 / sqrt(block_sum(q, red));           // its barriers also publish w_s
        constexpr int RW = kRowsPerWg / 4;                          // rows per wave, taken together
        double d[RW];
        const double* rowp[RW];
#pragma unroll
        for (int rr = 0; rr < RW; ++rr) {
            const int i = row0 + wave * RW + rr;
            d[rr] = 0.0;
            rowp[rr] = P + (size_t)(i < n ? i : n - 1) * r;        // a row beyond the end reads the last row, its result is dropped
        }
#pragma unroll 2
        for (int k = lane; k < r; k += 64) {
            const double wk = w_s[k];
#pragma unroll
            for (int rr = 0; rr < RW; ++rr) d[rr] = fma(fabs(rowp[rr][k]), wk, d[rr]);
        }
#pragma unroll
        for (int rr = 0; rr < RW; ++rr) {
            const int i = row0 + wave * RW + rr;
            const double v = wave_sum(d[rr]) * inv;
            if (lane == 0) {
                a_s[wave * RW + rr] = i < n ? v : 0.0;
                if (i < n) a_out[i] = v;
            }
        }
    } else if (tid < kRowsPerWg) {
        a_s[tid] = row0 + tid < n ? 1.0 : 0.0;
    }
    __syncthreads();
    if (rows_only) return;
    for (int k = tid; k < r; k += 256) {
        double c = 0.0;
#pragma unroll
        for (int rr = 0; rr < kRowsPerWg; ++rr) {
            const int i = row0 + rr;
            c = fma(fabs(P[(size_t)(i < n ? i : n - 1) * r + k]), a_s[rr], c);      // a_s = 0 beyond the end
        }
        partial[(size_t)blockIdx.x * r + k] = c;
    }
}

// w8[q][k] = sum over the parts g = q, q + 8, q + 16, ... of partial[g][k], added in index order by four threads per
// column whose results are combined in a fixed tree.
__global__ __launch_bounds__(256) void power_reduce_kernel(const double* partial, int n_parts, int r, double* w8)
{
    __shared__ double s[4][64];
    const int c = threadIdx.x & 63, t = threadIdx.x >> 6;
    const int k = blockIdx.x * 64 + c, q = blockIdx.y;
    double acc = 0.0;
    if (k < r)
        for (int g = q + kWParts * t; g < n_parts; g += kWParts * 4) acc += partial[(size_t)g * r + k];
    s[t][c] = acc;
    __syncthreads();
    if (t == 0 && k < r) w8[(size_t)q * r + k] = (s[0][c] + s[1][c]) + (s[2][c] + s[3][c]);
}

// Z = sign(P) (.) (a b^T) with b = w / ||w||  (power_iters = 0: the constant sum(w) / (n r), w = |P|^T 1),
// and the dual update in its two forms:  first = 0:  Lambda = P - Z  (P = X + Lambda_old, so this is
// Lambda_old + X - Z),  D = Z - Lambda;   first = 1 (initial state):  Lambda = 0,  D = Z.
__global__ __launch_bounds__(256) void svid_finish_kernel(const double* P, int n, int r, const double* a, const double* w8, int zero_rounds,
                                                           int first, double* Z, double* Lambda, double* D)
{
    extern __shared__ __align__(16) double w_s[];
    __shared__ double red[4];
    const int tid = threadIdx.x;
    double q = 0.0;
    for (int k = tid; k < r; k += 256) {
        const double v = w_at(w8, r, k);
        w_s[k] = v;
        q = zero_rounds ? q + v : fma(v, v, q);
    }
    const double tot = block_sum(q, red);
    const double scale = zero_rounds ? tot / ((double)n * (double)r) : 1.0 / sqrt(tot);
    const int row0 = blockIdx.x * kRowsPerWg;
    for (int k = tid; k < r; k += 256) {
        const double bk = zero_rounds ? scale : w_s[k] * scale;
#pragma unroll 4
        for (int rr = 0; rr < kRowsPerWg; ++rr) {
            const int i = row0 + rr;
            if (i >= n) break;
            const size_t e = (size_t)i * r + k;
            const double p = P[e];
            const double mag = zero_rounds ? scale : a[i] * bk;
            const double z = (p >= 0.0) ? mag : -mag;
            Z[e] = z;
            const double lam = first ? 0.0 : p - z;
            Lambda[e] = lam;
            D[e] = z - lam;
        }
    }
}

// ============================================================================================
//  Magnitude balancing (Step 2-3)
// ============================================================================================
__global__ __launch_bounds__(256) void sumsq_kernel(const double* X, const double* L, size_t count, double* partial)
{
    __shared__ double red[4];
    double q = 0.0;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < count; e += (size_t)gridDim.x * 256) {
        const double p = X[e] + L[e];
        q = fma(p, p, q);
    }
    const double t = block_sum(q, red);
    if (threadIdx.x == 0) partial[blockIdx.x] = t;
}

constexpr int kSumParts = 256;

// One wave per row: scale[i] = mean_k |f p_ik| with f = eta (which = 0) or 1 / eta (which = 1), p = X + L, and the
// packed sign bits of the row (bit = 1 iff p >= 0; a NaN packs as 0).
__global__ __launch_bounds__(256) void balance_rows_kernel(const double* X, const double* L, int rows, int r, const double* parts_u,
                                                            const double* parts_v, int which, uint32_t* words, double* scale, double* eta_out)
{
    __shared__ double red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double su = block_sum(parts_u[tid], red);
    const double sv = block_sum(parts_v[tid], red);
    const double eta = sqrt(sqrt(sv) / sqrt(su));
    if (eta_out && blockIdx.x == 0 && tid == 0) *eta_out = eta;
    const double f = which == 0 ? eta : 1.0 / eta;
    const int i = blockIdx.x * 4 + wave;
    if (i >= rows) return;
    const int n_words = (r + 31) / 32;
    double acc = 0.0;
    for (int c = 0; c * 64 < r; ++c) {
        const int k = c * 64 + lane;
        double p = -1.0;
        if (k < r) {
            p = X[(size_t)i * r + k] + L[(size_t)i * r + k];
            acc += fabs(f * p);
        }
        const unsigned long long bits = __ballot(k < r && p >= 0.0);
        if (lane == 0) {
            words[(size_t)i * n_words + 2 * c] = (uint32_t)bits;
            if (2 * c + 1 < n_words) words[(size_t)i * n_words + 2 * c + 1] = (uint32_t)(bits >> 32);
        }
    }
    acc = wave_sum(acc);
    if (lane == 0) scale[i] = acc / (double)r;
}

// ============================================================================================
//  Host side: workspace layout and the sequence of launches
// ============================================================================================
static int64_t next_pow2(int64_t v) { int64_t p = 1; while (p < v) p <<= 1; return p; }
static size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }

struct AdmmWs {
    int rp;            // padded side of the r x r matrices: 64 * 2^ceil(log2(ceil(r/64)))
    int rr;            // 64 * ceil(r/64): the part the factorisation touches
    double *H, *Linv, *Hinv, *T, *RHS, *P, *DU, *DV, *a, *w, *partial, *parts_u, *parts_v;
    double* G[3];      // three more [rp][rp] buffers for the parts of the Gram product's reduction (small ranks only, else nullptr)
    int* status;
    size_t bytes;
};

constexpr int kGramSixPartsMaxSide = 2048;

static AdmmWs carve(void* base, int64_t n, int64_t m, int64_t r)
{
    AdmmWs ws{};
    const int64_t q = (r + kNB - 1) / kNB;
    ws.rr = (int)(q * kNB);
    ws.rp = (int)(next_pow2(q) * kNB);
    const int64_t big = n > m ? n : m;
    size_t off = 0;
    auto take = [&](size_t count) { double* p = base ? (double*)((char*)base + off) : nullptr; off += up256(count * sizeof(double)); return p; };
    const size_t sq = (size_t)ws.rp * ws.rp;
    ws.H = take(sq); ws.Linv = take(sq); ws.Hinv = take(sq); ws.T = take(sq);
    // (a small Gram matrix has few tiles: its reduction is cut into six parts instead of three to fill the chip)
    for (double*& gp : ws.G) gp = ws.rp <= kGramSixPartsMaxSide ? take(sq) : nullptr;
    ws.RHS = take((size_t)big * r); ws.P = take((size_t)big * r);
    ws.DU = take((size_t)n * r); ws.DV = take((size_t)m * r);
    ws.a = take(big); ws.w = take((size_t)kWParts * r);
    ws.partial = take((size_t)((big + kRowsPerWg - 1) / kRowsPerWg) * r);
    ws.parts_u = take(kSumParts); ws.parts_v = take(kSumParts);
    ws.status = (int*)take(32);
    ws.bytes = off;
    return ws;
}

// SVID of P [rows][r] by `iters` rounds of power iteration; writes Z, Lambda and D = Z - Lambda.
static int svid(const AdmmWs& ws, const double* P, int rows, int r, int iters, int first, double* Z, double* Lambda, double* D, hipStream_t s)
{
    const int n_wg = (rows + kRowsPerWg - 1) / kRowsPerWg;
    const dim3 red_grid((r + 63) / 64, kWParts);
    const size_t lds = (size_t)r * sizeof(double);
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {        // r doubles of dynamic LDS plus the kernels' own few words can pass 64 KiB at the largest rank
        const int most = NQ_ADMM_MAX_RANK * (int)sizeof(double);
        attr_err = hipFuncSetAttribute((const void*)power_pass_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, most);
        if (attr_err == hipSuccess) attr_err = hipFuncSetAttribute((const void*)svid_finish_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, most);
    });
    NQ_HIP(attr_err);
    // w = |P|^T 1
    hipLaunchKernelGGL(power_pass_kernel, dim3(n_wg), dim3(256), lds, s, P, rows, r, (const double*)nullptr, 1, 0, ws.a, ws.partial);
    hipLaunchKernelGGL(power_reduce_kernel, red_grid, dim3(256), 0, s, ws.partial, n_wg, r, ws.w);
    for (int it = 0; it < iters; ++it) {
        // a = |P| b with b = w / ||w||; and, except in the last round, the next w = |P|^T a
        const int last = it + 1 == iters;
        hipLaunchKernelGGL(power_pass_kernel, dim3(n_wg), dim3(256), lds, s, P, rows, r, (const double*)ws.w, 0, last, ws.a, ws.partial);
        if (!last) hipLaunchKernelGGL(power_reduce_kernel, red_grid, dim3(256), 0, s, ws.partial, n_wg, r, ws.w);
    }
    hipLaunchKernelGGL(svid_finish_kernel, dim3(n_wg), dim3(256), lds, s, P, rows, r, (const double*)ws.a, (const double*)ws.w, iters == 0 ? 1 : 0, first,
                       Z, Lambda, D);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

// H (leading rr x rr of [rp][rp], lower part) -> L in place, Linv = L^-1, Hinv = L^-T L^-1.
static int factor_and_invert(const AdmmWs& ws, hipStream_t s, int prio)
{
    const int rp = ws.rp, rr = ws.rr, q = rr / kNB;
    static_assert(potrf_lds_bytes<kNB>() <= gemm_lds_bytes<64, 64>(), "the step kernel's LDS is the product's");
    const bool fused = !opt_flag(OPT_ADMM_NO_FUSED_STEP);
    constexpr size_t potrf_lds = potrf_lds_bytes<kNB>();
    constexpr size_t step_lds = gemm_lds_bytes<64, 64>();
    // where the blocks of L below the diagonal end up: a matrix of their own with the one-launch step (Hinv's buffer,
    // free until the last product below), in place of A21 with separate launches
    const double* const Lb = fused ? ws.Hinv : ws.H;
    hipLaunchKernelGGL(potrf_inv_kernel<kNB>, dim3(1), dim3((kNB / 4) * (kNB / 4)), potrf_lds, s, ws.H, rp, ws.Linv, rp, 0, ws.status, prio);
    for (int k = 0; k + 1 < q; ++k) {
        const int o = k * kNB;
        const int rem = rr - o - kNB;
        if (fused) {
            StepArgs sa{ws.H, ws.Hinv, ws.Linv, ws.T, rp, o, prio, ws.status};
            const int tiles = rem / kNB;
            hipLaunchKernelGGL(chol_step_kernel, dim3(tiles, tiles + 1), dim3(kGemmThreads), step_lds, s, sa);
            continue;
        }
        double* A21 = ws.H + (size_t)(o + kNB) * rp + o;
        // panel: L21 = A21 L11^-T, in place (a workgroup reads all of its rows before it writes them)
        GemmArgs p = gemm_args(0, 1, rem, kNB, kNB, 1.0, A21, rp, ws.Linv + (size_t)o * rp + o, rp, 0.0, nullptr, 0, A21, rp);
        p.tile = 3;                                // whole rows per workgroup: the product is in place
        p.prio = prio;
        int rc = launch_gemm(p, 1, s);
        if (rc != NQ_OK) return rc;
        // trailing update: A22 -= L21 L21^T (lower tiles only)
        double* A22 = ws.H + (size_t)(o + kNB) * rp + o + kNB;
        GemmArgs u = gemm_args(0, 1, rem, rem, kNB, -1.0, A21, rp, A21, rp, 1.0, A22, rp, A22, rp);
        u.lower_only = 1;
        u.prio = prio;
        rc = launch_gemm(u, 1, s);
        if (rc != NQ_OK) return rc;
        hipLaunchKernelGGL(potrf_inv_kernel<kNB>, dim3(1), dim3((kNB / 4) * (kNB / 4)), potrf_lds, s, ws.H, rp, ws.Linv, rp, o + kNB, ws.status, prio);
    }
    NQ_HIP(hipGetLastError());
    // L^-1 block-recursively: with the halves of a diagonal block inverted (X11, X22), the block below the
    // diagonal of its inverse is  -X22 L21 X11;  all pairs of one level run as one batched launch.
    for (int b = kNB; b < rr; b *= 2) {
        const int pairs = (rr - b + 2 * b - 1) / (2 * b);       // pairs whose lower half holds real rows
        const long long stride = (long long)2 * b * rp + 2 * b;
        GemmArgs t = gemm_args(0, 0, b, b, b, 1.0, Lb + (size_t)b * rp, rp, ws.Linv, rp, 0.0, nullptr, 0, ws.T + (size_t)b * rp, rp);
        t.sA = t.sB = t.sC = stride;
        t.prio = prio;
        int rc = launch_gemm(t, pairs, s);
        if (rc != NQ_OK) return rc;
        GemmArgs x = gemm_args(0, 0, b, b, b, -1.0, ws.Linv + (size_t)b * rp + b, rp, ws.T + (size_t)b * rp, rp, 0.0, nullptr, 0,
                               ws.Linv + (size_t)b * rp, rp);
        x.sA = x.sB = x.sC = stride;
        x.prio = prio;
        rc = launch_gemm(x, pairs, s);
        if (rc != NQ_OK) return rc;
    }
    GemmArgs h = gemm_args(1, 0, rr, rr, rr, 1.0, ws.Linv, rp, ws.Linv, rp, 0.0, nullptr, 0, ws.Hinv, rp);
    h.k_from_max = 1;
    h.prio = prio;
    return launch_gemm(h, 1, s);
}

// A second stream and three events, created once.  Two things run beside the factorisation, which is a chain of small
// launches that leaves most of the chip idle: the product with W (it does not depend on the factorisation), and the
// SVID of the factor just updated (nothing needs its result before that factor's NEXT update, a whole factor step later;
// the other factor's update only reads the new factor itself).
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr, updated = nullptr;
    hipError_t err = hipSuccess;
};

static SideStream& side_stream()
{
    static SideStream ss;
    static std::once_flag once;
    std::call_once(once, [] {
        ss.err = hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking);
        if (ss.err == hipSuccess) ss.err = hipEventCreateWithFlags(&ss.fork, hipEventDisableTiming);
        if (ss.err == hipSuccess) ss.err = hipEventCreateWithFlags(&ss.join, hipEventDisableTiming);
        if (ss.err == hipSuccess) ss.err = hipEventCreateWithFlags(&ss.updated, hipEventDisableTiming);
    });
    return ss;
}

// One factor update of Eq. 5 and Eq. 6 for X [rows][r] given the other factor O [cols][r]:
//   op(W) is [rows][cols] (w_trans = 1: W is stored [cols][rows]).
// An SVID whose launches are still to be issued (to the side stream): the factor step that follows issues them behind its
// own first launch, so that the host does not hold that launch -- the head of the critical path -- back by twenty others.
struct PendingSvid {
    bool valid = false;
    int rows = 0;
    double *Z = nullptr, *Lambda = nullptr, *D = nullptr;
};

static int issue_pending_svid(const AdmmWs& ws, PendingSvid& pend, int r, int power_iters)
{
    if (!pend.valid) return NQ_OK;
    pend.valid = false;
    SideStream& ss = side_stream();
    NQ_HIP(hipStreamWaitEvent(ss.stream, ss.updated, 0));
    return svid(ws, ws.P, pend.rows, r, power_iters, 0, pend.Z, pend.Lambda, pend.D, ss.stream);
}

static int factor_step(const AdmmWs& ws, const double* W, int w_trans, int ldw, int rows, int cols, int r, const double* O, double rho, double lam,
                       int power_iters, double* X, double* Z, double* Lambda, double* D, hipStream_t s, PendingSvid& pend)
{
    const bool overlap = !opt_flag(OPT_ADMM_NO_OVERLAP);
    // the launches of the caller's stream are the critical path: where another stream shares the chip, their waves
    // ask for the issue slots first
    const int prio = overlap && !opt_flag(OPT_ADMM_NO_PRIO);
    SideStream& ss = side_stream();
    NQ_HIP(ss.err);
    // H = O^T O + (rho + lambda) I   (lower tiles), its factor and inverse
    GemmArgs gh = gemm_args(1, 0, r, r, cols, 1.0, O, r, O, r, 0.0, nullptr, 0, ws.H, ws.rp);
    gh.diag = rho + lam;
    gh.lower_only = 1;
    gh.prio = prio;
    // a long reduction over few tiles: three or six parts of the reduction side by side (into H, two buffers that are
    // free at this point, and three of their own), then added in a fixed order
    // (small ranks: six parts on 128 x 128 tiles -- wider tiles halve what the tiles fetch between them, and the
    // parts make up for their number: 232 -> 190 us for r = 1024, 4096 rows)
    const bool six = ws.G[0] && cols >= 1536 && r >= 256;
    const int parts = cols >= 768 ? (six ? 6 : 3) : 1;
    if (parts > 1) {
        gh.k_parts = parts;
        gh.k_per_part = ((cols + parts - 1) / parts + kBK - 1) / kBK * kBK;
        gh.Cp[0] = ws.H; gh.Cp[1] = ws.T; gh.Cp[2] = ws.Hinv;
        gh.Cp[3] = ws.G[0]; gh.Cp[4] = ws.G[1]; gh.Cp[5] = ws.G[2];
    }
    if (six) gh.tile = 1;
    int rc = launch_gemm(gh, parts, s);
    if (rc != NQ_OK) return rc;
    if (parts > 1) {
        GramParts gp{};
        gp.n = parts;
        for (int q = 0; q < parts; ++q) gp.p[q] = gh.Cp[q];
        hipLaunchKernelGGL(add_parts_kernel, dim3((r + 255) / 256, r), dim3(256), 0, s, ws.H, gp, ws.rp, r);
        NQ_HIP(hipGetLastError());
    }
    rc = issue_pending_svid(ws, pend, r, power_iters);        // the other factor's SVID, to the side stream
    if (rc != NQ_OK) return rc;
    // RHS = op(W) O + rho (Z - Lambda), on the side stream (behind the SVID that produced Z and Lambda).  It is let go
    // once the Gram matrix is done: both fill the chip, so side by side neither gains, and the product would only keep
    // the Gram matrix -- the head of the critical path -- waiting for workgroup slots; what the product can hide behind
    // is the factorisation that follows.
    hipStream_t rs = overlap ? ss.stream : s;
    if (overlap) {
        NQ_HIP(hipEventRecord(ss.fork, s));
        NQ_HIP(hipStreamWaitEvent(ss.stream, ss.fork, 0));
    }
    GemmArgs gr = gemm_args(w_trans, 0, rows, r, cols, 1.0, W, ldw, O, r, rho, D, r, ws.RHS, r);
    // On its own (everything on one stream) the product wants the 128 x 128 tile with two workgroups per CU: where the
    // output has fewer tiles than that, the reduction is cut in two halves (the second into P's buffer, which is free
    // until the solve) and the halves are added.
    // Beside the factorisation it is the other way round: the product has the whole factorisation to finish in, and what
    // matters is that the factorisation's small launches find room at once -- with two 128 x 128 workgroups on a CU
    // (2 x 72 KiB of LDS) a 64 x 64 workgroup (40 KiB) has to wait until one of them has finished its whole reduction
    // (measured: a panel update of 15 workgroups took 470-570 us instead of 8).  So the product then runs with at
    // most ONE workgroup per CU (its LDS request is padded past half a CU's) and without the cut.
    const long long t128 = (long long)((rows + 127) / 128) * ((r + 127) / 128);
    const bool roomy = overlap && opt_or(OPT_ADMM_PRODUCT_MODE, 0) != 1 && t128 >= 64;
    const int w_parts = !roomy && t128 < 512 && 2 * t128 >= 384 && cols >= 1024 ? 2 : 1;
    if (w_parts > 1) {
        gr.k_parts = 2;
        gr.k_per_part = ((cols + 1) / 2 + kBK - 1) / kBK * kBK;
        gr.Cp[0] = ws.RHS; gr.Cp[1] = ws.P;
    }
    if (roomy) {
        gr.tile = 1;
        gr.lds_pad = 16384;
    }
    rc = launch_gemm(gr, w_parts, rs);
    if (rc != NQ_OK) return rc;
    if (w_parts > 1) {
        hipLaunchKernelGGL(add_half_kernel, dim3(1024), dim3(256), 0, rs, ws.RHS, (const double*)ws.P, (size_t)rows * r);
        NQ_HIP(hipGetLastError());
    }
    if (overlap) NQ_HIP(hipEventRecord(ss.join, ss.stream));
    rc = factor_and_invert(ws, s, prio);
    if (rc != NQ_OK) return rc;
    if (overlap) NQ_HIP(hipStreamWaitEvent(s, ss.join, 0));
    // X = RHS H^-1,  P = X + Lambda
    GemmArgs gx = gemm_args(0, 0, rows, r, r, 1.0, ws.RHS, r, ws.Hinv, ws.rp, 0.0, nullptr, 0, X, r);
    gx.E = Lambda;
    gx.C2 = ws.P;
    gx.prio = prio;
    rc = launch_gemm(gx, 1, s);
    if (rc != NQ_OK) return rc;
    if (!overlap || opt_flag(OPT_ADMM_INLINE_SVID)) return svid(ws, ws.P, rows, r, power_iters, 0, Z, Lambda, D, s);
    // The SVID goes to the side stream.  What keeps the buffers apart: the side stream runs SVID (reads P; writes Z,
    // Lambda, D), then the next factor step's product (second half into P, result into RHS), in that order; the
    // caller's stream writes P and reads RHS and Lambda only after it has waited for that product.
    // (Its launches are issued by the next factor step, or by the caller after the last one.)
    NQ_HIP(hipEventRecord(ss.updated, s));
    pend.valid = true;
    pend.rows = rows; pend.Z = Z; pend.Lambda = Lambda; pend.D = D;
    return NQ_OK;
}

static int fail(int code, const char* msg)
{
    set_error(msg);
    return code;
}

static bool aligned8(const void* p) { return ((uintptr_t)p & 7u) == 0; }

static int check_shape(int64_t n, int64_t m, int64_t r)
{
    if (n < 1 || m < 1 || r < 1) return fail(NQ_E_SHAPE, "lb_admm: n, m, r must be >= 1");
    if (n > NQ_ADMM_MAX_DIM || m > NQ_ADMM_MAX_DIM || r > NQ_ADMM_MAX_RANK) return fail(NQ_E_SHAPE, "lb_admm: n, m or r beyond the supported size");
    if ((uint64_t)n * (uint64_t)m >= (1ull << 40)) return fail(NQ_E_SHAPE, "lb_admm: n * m too large");
    return NQ_OK;
}

}  // namespace nq

using namespace nq;

extern "C" int nq_lb_admm_workspace_bytes(int64_t n, int64_t m, int64_t r, size_t* bytes)
{
    if (!bytes) return fail(NQ_E_NULL, "lb_admm_workspace_bytes: bytes is NULL");
    const int rc = check_shape(n, m, r);
    if (rc != NQ_OK) return rc;
    *bytes = carve(nullptr, n, m, r).bytes;
    return NQ_OK;
}

extern "C" int nq_lb_admm(const double* W, int64_t n, int64_t m, int64_t r, const double* U0, const double* V0, int n_iters, double rho_start,
                          double rho_end, double lambda, int power_iters, double* U, double* V, double* Z_U, double* Z_V, double* Lambda_U,
                          double* Lambda_V, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!W || !U0 || !V0 || !U || !V || !Z_U || !Z_V || !Lambda_U || !Lambda_V || !workspace) return fail(NQ_E_NULL, "lb_admm: NULL pointer");
    int rc = check_shape(n, m, r);
    if (rc != NQ_OK) return rc;
    const void* ptrs[] = {W, U0, V0, U, V, Z_U, Z_V, Lambda_U, Lambda_V};
    for (const void* p : ptrs)
        if (!aligned8(p)) return fail(NQ_E_ALIGN, "lb_admm: a matrix pointer is not 8-byte aligned");
    if (((uintptr_t)workspace & 255u) != 0) return fail(NQ_E_ALIGN, "lb_admm: workspace is not 256-byte aligned");
    if (n_iters < 0 || power_iters < 0) return fail(NQ_E_INVALID_ARG, "lb_admm: n_iters and power_iters must be >= 0");
    if (!isfinite(rho_start) || !isfinite(rho_end) || !isfinite(lambda)) return fail(NQ_E_INVALID_ARG, "lb_admm: rho and lambda must be finite");
    const AdmmWs ws = carve(workspace, n, m, r);
    if (workspace_bytes < ws.bytes) return fail(NQ_E_INVALID_ARG, "lb_admm: workspace smaller than nq_lb_admm_workspace_bytes");
    hipStream_t s = (hipStream_t)stream;
    const int N = (int)n, M = (int)m, R = (int)r;

    NQ_HIP(hipMemsetAsync(ws.status, 0, 256, s));
    hipLaunchKernelGGL(pad_identity_kernel, dim3(256), dim3(256), 0, s, ws.H, ws.rp, R, 0);
    hipLaunchKernelGGL(pad_identity_kernel, dim3(256), dim3(256), 0, s, ws.Linv, ws.rp, R, 1);
    NQ_HIP(hipGetLastError());
    if (U != U0) NQ_HIP(hipMemcpyAsync(U, U0, (size_t)n * r * sizeof(double), hipMemcpyDeviceToDevice, s));
    if (V != V0) NQ_HIP(hipMemcpyAsync(V, V0, (size_t)m * r * sizeof(double), hipMemcpyDeviceToDevice, s));
    // initial state: Z = SVID of the start factors, Lambda = 0
    rc = svid(ws, U, N, R, power_iters, 1, Z_U, Lambda_U, ws.DU, s);
    if (rc != NQ_OK) return rc;
    rc = svid(ws, V, M, R, power_iters, 1, Z_V, Lambda_V, ws.DV, s);
    if (rc != NQ_OK) return rc;
    PendingSvid pend;
    for (int k = 0; k < n_iters; ++k) {
        const double rho = n_iters <= 1 ? rho_start : rho_start + (rho_end - rho_start) * (double)k / (double)(n_iters - 1);
        rc = factor_step(ws, W, 0, M, N, M, R, V, rho, lambda, power_iters, U, Z_U, Lambda_U, ws.DU, s, pend);
        if (rc != NQ_OK) return rc;
        rc = factor_step(ws, W, 1, M, M, N, R, U, rho, lambda, power_iters, V, Z_V, Lambda_V, ws.DV, s, pend);
        if (rc != NQ_OK) return rc;
    }
    rc = issue_pending_svid(ws, pend, R, power_iters);
    if (rc != NQ_OK) return rc;
    if (n_iters > 0 && !opt_flag(OPT_ADMM_NO_OVERLAP)) {      // the last SVID may still be running on the side stream
        SideStream& ss = side_stream();
        NQ_HIP(hipEventRecord(ss.join, ss.stream));
        NQ_HIP(hipStreamWaitEvent(s, ss.join, 0));
    }
    int status = 0;
    NQ_HIP(hipMemcpyAsync(&status, ws.status, sizeof(int), hipMemcpyDeviceToHost, s));
    NQ_HIP(hipStreamSynchronize(s));
    if (status != 0) return fail(NQ_E_INVALID_ARG, "lb_admm: a pivot of the Cholesky factorisation was not positive (rho + lambda <= 0, or NaN in the input)");
    return NQ_OK;
}

extern "C" int nq_lb_admm_balance(const double* U, const double* Lambda_U, int64_t n, const double* V, const double* Lambda_V, int64_t m, int64_t r,
                                  uint32_t* U_words, uint32_t* V_words, double* s1, double* s2, double* eta, void* workspace,
                                  size_t workspace_bytes, void* stream)
{
    if (!U || !Lambda_U || !V || !Lambda_V || !U_words || !V_words || !s1 || !s2 || !eta || !workspace) return fail(NQ_E_NULL, "lb_admm_balance: NULL pointer");
    const int rc = check_shape(n, m, r);
    if (rc != NQ_OK) return rc;
    const void* ptrs[] = {U, Lambda_U, V, Lambda_V, s1, s2, eta};
    for (const void* p : ptrs)
        if (!aligned8(p)) return fail(NQ_E_ALIGN, "lb_admm_balance: a pointer is not 8-byte aligned");
    if (((uintptr_t)U_words & 3u) || ((uintptr_t)V_words & 3u)) return fail(NQ_E_ALIGN, "lb_admm_balance: word pointers must be 4-byte aligned");
    if (((uintptr_t)workspace & 255u) != 0) return fail(NQ_E_ALIGN, "lb_admm_balance: workspace is not 256-byte aligned");
    const AdmmWs ws = carve(workspace, n, m, r);
    if (workspace_bytes < ws.bytes) return fail(NQ_E_INVALID_ARG, "lb_admm_balance: workspace smaller than nq_lb_admm_workspace_bytes");
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(sumsq_kernel, dim3(kSumParts), dim3(256), 0, s, U, Lambda_U, (size_t)n * r, ws.parts_u);
    hipLaunchKernelGGL(sumsq_kernel, dim3(kSumParts), dim3(256), 0, s, V, Lambda_V, (size_t)m * r, ws.parts_v);
    hipLaunchKernelGGL(balance_rows_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, s, U, Lambda_U, (int)n, (int)r, (const double*)ws.parts_u,
                       (const double*)ws.parts_v, 0, U_words, s1, eta);
    hipLaunchKernelGGL(balance_rows_kernel, dim3((unsigned)((m + 3) / 4)), dim3(256), 0, s, V, Lambda_V, (int)m, (int)r, (const double*)ws.parts_u,
                       (const double*)ws.parts_v, 1, V_words, s2, (double*)nullptr);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

extern "C" int nq_dgemm(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K, double alpha, const double* A, int64_t lda, const double* B,
                        int64_t ldb, double beta, double* C, int64_t ldc, void* stream)
{
    if (!A || !B || !C) return fail(NQ_E_NULL, "dgemm: NULL pointer");
    if (M < 1 || N < 1 || K < 1 || M > NQ_ADMM_MAX_DIM || N > NQ_ADMM_MAX_DIM || K > NQ_ADMM_MAX_DIM) return fail(NQ_E_SHAPE, "dgemm: M, N, K must be in [1, 65536]");
    if ((trans_a | trans_b) & ~1) return fail(NQ_E_INVALID_ARG, "dgemm: trans flags are 0 or 1");
    if (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N) || ldc < N || lda > INT32_MAX || ldb > INT32_MAX || ldc > INT32_MAX)
        return fail(NQ_E_SHAPE, "dgemm: a leading dimension is smaller than its row length");
    if (!aligned8(A) || !aligned8(B) || !aligned8(C)) return fail(NQ_E_ALIGN, "dgemm: a pointer is not 8-byte aligned");
    GemmArgs g = gemm_args(trans_a, trans_b, (int)M, (int)N, (int)K, alpha, A, (int)lda, B, (int)ldb, beta, C, (int)ldc, C, (int)ldc);
    return launch_gemm(g, 1, (hipStream_t)stream);
}
