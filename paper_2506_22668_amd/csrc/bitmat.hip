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
// out[i] = sum over set bits j of row i of x[j]; one wave per row, lanes over words.
__global__ __launch_bounds__(kThreads) void bit_spmv_kernel(const uint64_t* B, int64_t rows, int64_t cols, int64_t stride,
                                                            int64_t row_first, int64_t row_step, const double* x,
                                                            double* out) {
  const int64_t Wc = (cols + 63) / 64;
  const uint64_t tail = (cols & 63) ? ((1ull << (cols & 63)) - 1ull) : ~0ull;
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t i = wave; i < rows; i += nwaves) {
    const uint64_t* row = B + (row_first + i * row_step) * stride;
    double acc = 0.0;
    for (int64_t wd = lane; wd < Wc; wd += 64) {
      uint64_t word = row[wd] & (wd == Wc - 1 ? tail : ~0ull);  // padding bits name no column
      const double* xb = x + wd * 64;
      while (word) {
        acc += xb[__ffsll((long long)word) - 1];
        word &= word - 1;
      }
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) out[i] = acc;
  }
}

}  // namespace

int ds_bit_spmv(ds_ctx* ctx, const uint64_t* B, int64_t rows, int64_t cols, int64_t stride, int64_t row_first,
                int64_t row_step, const double* x, double* out) {
  if (rows <= 0) return DS_OK;
  int64_t blocks = (rows * 64 + kThreads - 1) / kThreads;
  if (blocks > (int64_t)ctx->num_cus * 8) blocks = (int64_t)ctx->num_cus * 8;
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
