// Helpers on bit-packed mask matrices shared by the two solvers: per-row
// regression targets and the bit-matrix transpose.
#include "internal.h"
#include "solve_common.h"

namespace {
constexpr int kThreads = 256;

// One wave per row: size |S_i| = popcount, target t_i = y_i - y_0 - (delta/n)|S_i|
// (the regression re-centred on the efficiency constraint), sqrt(w_i), and w_i itself
// with the two constraint rows zeroed.
__global__ __launch_bounds__(kThreads) void row_prep_kernel(const uint64_t* Z, int64_t k, int64_t W, int64_t n,
                                                            const float* w, const float* y, int32_t* sz, double* t,
                                                            double* sqw, float* wc) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const double f0 = (double)y[0], delta = (double)y[1] - (double)y[0];
  for (int64_t i = wave; i < k; i += nwaves) {
    int c = 0;
    const uint64_t tail = (n & 63) ? ((1ull << (n & 63)) - 1ull) : ~0ull;
    for (int64_t wd = lane; wd < W; wd += 64) c += __popcll(Z[i * W + wd] & (wd == W - 1 ? tail : ~0ull));
    for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
    if (lane == 0) {
      sz[i] = c;
      t[i] = i < 2 ? 0.0 : (double)y[i] - f0 - (delta / (double)n) * (double)c;
      sqw[i] = i < 2 ? 0.0 : sqrt((double)w[i]);
      wc[i] = i < 2 ? 0.f : w[i];
    }
  }
}

// Transpose a bit matrix: in[rows x Win words] (row stride in_stride words, rows taken
// as row_first + i*row_step) -> out[cols x Wout words], Wout = ceil(rows/64); bit i of
// out row j = bit j of in row i. One wave per 64x64 block: lane l loads the word of
// row l; ballot j collects bit j of all 64 rows, which is the word of column j.
__global__ __launch_bounds__(kThreads) void bit_transpose_kernel(const uint64_t* in, int64_t rows, int64_t cols,
                                                                 int64_t in_stride, int64_t row_first, int64_t row_step,
                                                                 uint64_t* out, int64_t Wout) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const int64_t Win = (cols + 63) / 64;
  const int64_t blocks = Wout * Win;
  for (int64_t b = wave; b < blocks; b += nwaves) {
    const int64_t rb = b / Win, cb = b - rb * Win;  // consecutive waves walk along a row block: coalesced reads
    const int64_t i = rb * 64 + lane;
    uint64_t word = 0;
    if (i < rows) word = in[(row_first + i * row_step) * in_stride + cb];
    uint64_t mine = 0;
#pragma unroll 8
    for (int j = 0; j < 64; ++j) {
      const uint64_t col = __ballot((word >> j) & 1ull);
      if (lane == j) mine = col;
    }
    const int64_t c = cb * 64 + lane;
    if (c < cols) out[c * Wout + rb] = mine;
  }
}
// out[i] = sum over the set bits j of row i of x[j] (fp64).
// The vector is staged through LDS in chunks of 8192 columns, so the one gather per set bit is an
// LDS read instead of an L2 transaction; the matrix is streamed once, each (row, chunk) segment
// being 1 KB of contiguous words. A wave owns 16 rows and keeps their partial sums in registers
// across all chunks (one cross-lane reduction per row at the very end); per chunk it first loads
// the two words of each of its rows into registers (16 independent row loads in flight), then walks
// their set bits. The LDS copy is pitched 65 doubles per 64-column word to spread the banks.
constexpr int kSpmvChunkWords = 128;
constexpr int kSpmvRowsPerWave = 16;
constexpr int kSpmvPitch = 65;

__global__ __launch_bounds__(kThreads) void bit_spmv_kernel(const uint64_t* B, int64_t rows, int64_t cols, int64_t stride,
                                                            int64_t row_first, int64_t row_step, const double* x,
                                                            double* out) {
  __shared__ double xs[kSpmvChunkWords * kSpmvPitch];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t Wc = (cols + 63) / 64;
  const uint64_t tail = (cols & 63) ? ((1ull << (cols & 63)) - 1ull) : ~0ull;
  // blocks walk the rows from the end: mask rows are sorted by size, so the long (dense) rows start first
  const int64_t row0 = (int64_t)(gridDim.x - 1 - blockIdx.x) * (kSpmvRowsPerWave * (kThreads / 64)) + (int64_t)wave * kSpmvRowsPerWave;
  double acc[kSpmvRowsPerWave];
#pragma unroll
  for (int i = 0; i < kSpmvRowsPerWave; ++i) acc[i] = 0.0;
  const double* xa = xs + (2 * lane) * kSpmvPitch;
  const double* xb = xs + (2 * lane + 1) * kSpmvPitch;
  for (int64_t c0 = 0; c0 < Wc; c0 += kSpmvChunkWords) {
    __syncthreads();
    for (int i = tid; i < kSpmvChunkWords * 64; i += kThreads) {
      const int64_t col = c0 * 64 + i;
      xs[(i >> 6) * kSpmvPitch + (i & 63)] = col < cols ? x[col] : 0.0;
    }
    __syncthreads();
    const int64_t wa = c0 + 2 * lane, wb = wa + 1;
    uint64_t w0[kSpmvRowsPerWave], w1[kSpmvRowsPerWave];
#pragma unroll
    for (int i = 0; i < kSpmvRowsPerWave; ++i) {
      const int64_t r = row0 + i;
      w0[i] = 0ull;
      w1[i] = 0ull;
      if (r < rows) {
        const uint64_t* p = B + (row_first + r * row_step) * stride;
        if (wa < Wc) w0[i] = p[wa] & (wa == Wc - 1 ? tail : ~0ull);  // padding bits name no column
        if (wb < Wc) w1[i] = p[wb] & (wb == Wc - 1 ? tail : ~0ull);
      }
    }
    // four rows (eight words) are walked together so that eight LDS reads are in flight
#pragma unroll
    for (int i = 0; i < kSpmvRowsPerWave; i += 4) {
      uint64_t m[8] = {w0[i], w1[i], w0[i + 1], w1[i + 1], w0[i + 2], w1[i + 2], w0[i + 3], w1[i + 3]};
      double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      while (m[0] | m[1] | m[2] | m[3] | m[4] | m[5] | m[6] | m[7]) {
        double v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const bool live = m[q] != 0ull;
          const int bit = live ? __ffsll((long long)m[q]) - 1 : 0;
          const double xv = (q & 1) ? xb[bit] : xa[bit];
          v[q] = live ? xv : 0.0;
          m[q] &= m[q] - 1;  // 0 stays 0
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) s[q] += v[q];
      }
      acc[i] += s[0] + s[1];
      acc[i + 1] += s[2] + s[3];
      acc[i + 2] += s[4] + s[5];
      acc[i + 3] += s[6] + s[7];
    }
  }
#pragma unroll
  for (int i = 0; i < kSpmvRowsPerWave; ++i) {
    double s = acc[i];
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0 && row0 + i < rows) out[row0 + i] = s;
  }
}

}  // namespace

int ds_bit_spmv(ds_ctx* ctx, const uint64_t* B, int64_t rows, int64_t cols, int64_t stride, int64_t row_first,
                int64_t row_step, const double* x, double* out) {
  if (rows <= 0) return DS_OK;
  const int64_t rows_per_block = kSpmvRowsPerWave * (kThreads / 64);
  const int64_t blocks = (rows + rows_per_block - 1) / rows_per_block;
  hipLaunchKernelGGL(bit_spmv_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, ctx->stream, B, rows, cols, stride,
                     row_first, row_step, x, out);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

int ds_row_prep(ds_ctx* ctx, const uint64_t* Z, int64_t k, int64_t n, const float* w, const float* y, int32_t* sz,
                double* t, double* sqw, float* wc) {
  const int64_t W = (n + 63) / 64;
  int64_t blocks = (k * 64 + kThreads - 1) / kThreads;
  if (blocks > (int64_t)ctx->num_cus * 16) blocks = (int64_t)ctx->num_cus * 16;
  hipLaunchKernelGGL(row_prep_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, ctx->stream, Z, k, W, n, w, y, sz, t, sqw, wc);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

int ds_bit_transpose(ds_ctx* ctx, const uint64_t* in, int64_t rows, int64_t cols, int64_t in_stride, int64_t row_first,
                     int64_t row_step, uint64_t* out) {
  const int64_t Wout = (rows + 63) / 64, Win = (cols + 63) / 64;
  int64_t blocks = (Wout * Win * 64 + kThreads - 1) / kThreads;
  if (blocks > (int64_t)ctx->num_cus * 16) blocks = (int64_t)ctx->num_cus * 16;
  if (blocks < 1) return DS_OK;
  hipLaunchKernelGGL(bit_transpose_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, ctx->stream, in, rows, cols,
                     in_stride, row_first, row_step, out, Wout);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}
