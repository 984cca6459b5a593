// Products with the TRANSPOSED sign matrices from the resident tiles of a layer (the training-time siblings of the
// forward: Section 3.4 and Algorithm 1, Phase 3 need  V (U^T (s_out (.) g))  for the gradient of the input scales).
// No second copy of the bits is made.  Inside a 128 x 64 tile a lane owns 16 columns and, of each, the 8 rows
// 16 p + (lane & 15): a column's rows are spread over 16 lanes, which no matrix instruction reduces over, so this path
// adds on the vector ALU in binary64 (exact sign products, one rounding when the result is stored).
#include "nq_internal.h"
#include "nq_device.h"

namespace nq {

constexpr int kTWaves = 4;

// partial[(sp * batch + tok) * n_pad + col] = sum over the row blocks rb = 4 sp + wave (mod 4 n_split) of
//     sum_row sign(row, col) * in_scale[row] * in[tok][row]
__global__ __launch_bounds__(64 * kTWaves) void gemv_t_kernel(const uint32_t* __restrict__ tiles, int nsteps, int n_rb, int M,
                                                              const void* __restrict__ in, int in_dtype, int in_stride,
                                                              const uint16_t* __restrict__ in_scale, double* __restrict__ partial,
                                                              int n_split, int batch)
{
    __shared__ double red[kTWaves][kTileCols];
    const int st = blockIdx.x, sp = blockIdx.y, tok = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ri = lane & 15, cg = lane >> 4;
    double acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.0;
    for (int rb = sp * kTWaves + wave; rb < n_rb; rb += kTWaves * n_split) {
        const v4u wd = *(const v4u*)(tiles + ((size_t)rb * nsteps + st) * kTileWords + 4 * lane);
        const uint32_t w[4] = {wd.x, wd.y, wd.z, wd.w};
        double x[8];
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int row = rb * kTileRows + 16 * p + ri;
            double v = 0.0;                                        // rows beyond M hold 0 bits and contribute nothing
            if (row < M) {
                v = (double)load_as_float(in, in_dtype, (size_t)tok * in_stride + row);
                if (in_scale) v *= (double)half_bits_to_float(in_scale[row]);
            }
            x[p] = v;
        }
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int p = 0; p < 8; ++p) acc[4 * v + b] += ((w[v] >> (8 * b + p)) & 1u) ? x[p] : -x[p];
    }
    // the 16 lanes of a column group hold the 16 row offsets of the same columns
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        double s = acc[j];
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) s += __shfl_xor(s, off);
        if (ri == 0) red[wave][16 * cg + j] = s;
    }
    __syncthreads();
    if (threadIdx.x < kTileCols) {
        const int c = threadIdx.x;
        const double s = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
        partial[((size_t)sp * batch + tok) * ((size_t)nsteps * kTileCols) + (size_t)st * kTileCols + c] = s;
    }
}

// out[tok][col] = out_scale[col] * sum_sp partial[sp][tok][col]   (splits added in index order)
__global__ __launch_bounds__(256) void gemv_t_finish_kernel(const double* __restrict__ partial, int n_split, int batch, int n_pad, int N,
                                                            const uint16_t* __restrict__ out_scale, void* __restrict__ out, int out_dtype,
                                                            int out_stride)
{
    const int col = blockIdx.x * 256 + threadIdx.x, tok = blockIdx.y;
    if (col >= N) return;
    double s = 0.0;
    for (int sp = 0; sp < n_split; ++sp) s += partial[((size_t)sp * batch + tok) * n_pad + col];
    if (out_scale) s *= (double)half_bits_to_float(out_scale[col]);
    store_out(out, out_dtype, (size_t)tok * out_stride + col, (float)s);
}

int gemv_t_splits(int64_t M, int64_t N, int batch)
{
    const int n_rb = (int)n_rowblocks(M), nst = (int)n_steps(N);
    int want = 512 / (nst * batch > 0 ? nst * batch : 1);
    const int most = n_rb / kTWaves > 0 ? n_rb / kTWaves : 1;
    if (want > most) want = most;
    if (want > 8) want = 8;
    return want < 1 ? 1 : want;
}

size_t gemv_t_partial_bytes(int64_t M, int64_t N, int batch)
{
    return (size_t)gemv_t_splits(M, N, batch) * batch * (size_t)n_steps(N) * kTileCols * sizeof(double);
}

// A is [M][N] as sign tiles; out[tok][0..N) = out_scale (.) A^T (in_scale (.) in[tok][0..M)).  `partial`: device,
// gemv_t_partial_bytes(M, N, batch).
int launch_gemv_t(const uint32_t* tiles, int64_t M, int64_t N, const void* in, int in_dtype, int in_stride, const uint16_t* in_scale,
                  const uint16_t* out_scale, void* out, int out_dtype, int out_stride, int batch, double* partial, hipStream_t s)
{
    const int n_rb = (int)n_rowblocks(M), nst = (int)n_steps(N), n_split = gemv_t_splits(M, N, batch);
    hipLaunchKernelGGL(gemv_t_kernel, dim3(nst, n_split, batch), dim3(64 * kTWaves), 0, s, tiles, nst, n_rb, (int)M, in, in_dtype, in_stride,
                       in_scale, partial, n_split, batch);
    hipLaunchKernelGGL(gemv_t_finish_kernel, dim3((unsigned)((N + 255) / 256), batch), dim3(256), 0, s, (const double*)partial, n_split, batch,
                       nst * kTileCols, (int)N, out_scale, out, out_dtype, out_stride);
    NQ_HIP(hipGetLastError());
    return NQ_OK;
}

}  // namespace nq
