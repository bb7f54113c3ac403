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


// Few rows (the tiled kernel above would leave most of the GPU idle): one wave per row, lanes over words.
__global__ __launch_bounds__(kThreads) void bit_spmv_rows_kernel(const uint64_t* B, int64_t rows, int64_t cols, int64_t stride,
                                                                 int64_t row_first, int64_t row_step, const double* x,
                                                                 double* out) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const int64_t Wc = (cols + 63) / 64;
  const uint64_t tail = (cols & 63) ? ((1ull << (cols & 63)) - 1ull) : ~0ull;
  for (int64_t i = wave; i < rows; i += nwaves) {
    const uint64_t* row = B + (row_first + i * row_step) * stride;
    double acc = 0.0;
    for (int64_t wd = lane; wd < Wc; wd += 128) {
      uint64_t w0 = row[wd] & (wd == Wc - 1 ? tail : ~0ull);
      uint64_t w1 = wd + 64 < Wc ? (row[wd + 64] & (wd + 64 == Wc - 1 ? tail : ~0ull)) : 0ull;
      const double* x0 = x + wd * 64;
      const double* x1 = x0 + 64 * 64;
      double a0 = 0.0, a1 = 0.0;
      while (w0 | w1) {  // four bits of either word per step: eight gathers in flight (same order of additions)
        double v0[4], v1[4];
        bool l0[4], l1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          l0[u] = w0 != 0ull;
          l1[u] = w1 != 0ull;
          v0[u] = x0[l0[u] ? __ffsll((long long)w0) - 1 : 0];
          v1[u] = *(l1[u] ? x1 + (__ffsll((long long)w1) - 1) : x0);  // x1 may lie past the end when w1 is empty
          w0 &= w0 - 1;
          w1 &= w1 - 1;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          a0 += l0[u] ? v0[u] : 0.0;
          a1 += l1[u] ? v1[u] : 0.0;
        }
      }
      acc += a0 + a1;
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) out[i] = acc;
  }
}

// ---- dense rows: byte-table product -------------------------------------------------------
// out[i] = sum over set bits j of row i of x[j], for rows that are dense enough that walking
// bits one by one costs more than it should. For a chunk of 512 columns the workgroup builds,
// in LDS, the 64 tables T_g[b] = sum of x over the bits of byte value b within column group g
// (from two 16-entry nibble tables per group), and every thread then adds eight table entries
// per 64-bit word of its rows: one LDS read per 8 matrix bits, whatever the density. A
// workgroup covers 2048 rows x a range of chunks; the per-range partial sums are added up in a
// fixed order by a second kernel.
constexpr int kTabCols = 512;
constexpr int kTabWords = kTabCols / 64;
constexpr int kTabGroups = kTabCols / 8;
constexpr int kTabThreads = 1024;  // 16 waves hide the LDS and memory latency of the look-ups
constexpr int kTabRpt = 4;         // rows per thread
constexpr int kTabRows = kTabThreads * kTabRpt;

__global__ __launch_bounds__(kTabThreads) void bit_spmv_tab_kernel(const uint64_t* B, int64_t rows, int64_t cols, int64_t stride,
                                                                int64_t row_first, int64_t row_step, const double* x,
                                                                double* partial, int64_t chunks_per_group, int64_t n_chunks) {
  extern __shared__ double tab_smem[];
  double* tab = tab_smem;                       // [64 groups][256]
  double* nib = tab_smem + kTabGroups * 256;    // [64 groups][2 nibbles][16]
  double* xch = nib + kTabGroups * 32;          // [512] the chunk of x
  const int tid = threadIdx.x;
  const int64_t Wc = (cols + 63) / 64;
  const uint64_t tail = (cols & 63) ? ((1ull << (cols & 63)) - 1ull) : ~0ull;
  const int64_t rbase = (int64_t)blockIdx.x * kTabRows;
  double acc[kTabRpt];
#pragma unroll
  for (int i = 0; i < kTabRpt; ++i) acc[i] = 0.0;
  const int64_t c_begin = (int64_t)blockIdx.y * chunks_per_group;
  const int64_t c_end = c_begin + chunks_per_group < n_chunks ? c_begin + chunks_per_group : n_chunks;
  for (int64_t c = c_begin; c < c_end; ++c) {
    __syncthreads();
    // the chunk's 512 vector entries first (one coalesced load), then the nibble sums from LDS
    if (tid < kTabCols) {
      const int64_t col = c * kTabCols + tid;
      xch[tid] = col < cols ? x[col] : 0.0;
    }
    __syncthreads();
    for (int e = tid; e < kTabGroups * 32; e += kTabThreads) {
      const int g = e >> 5, half = (e >> 4) & 1, m = e & 15;
      const double* xp = xch + g * 8 + half * 4;
      double sum = 0.0;
#pragma unroll
      for (int bbit = 0; bbit < 4; ++bbit)
        if ((m >> bbit) & 1) sum += xp[bbit];
      nib[e] = sum;
    }
    __syncthreads();
    for (int e = tid; e < kTabGroups * 256; e += kTabThreads) {
      const int g = e >> 8, byte = e & 255;
      tab[e] = nib[g * 32 + (byte & 15)] + nib[g * 32 + 16 + (byte >> 4)];
    }
    __syncthreads();
    // all words of the thread's rows for this chunk are requested first (their latency overlaps);
    // then, word by word, the eight table reads are issued together and summed as a tree, so that
    // the LDS pipeline stays full instead of waiting on one read at a time
    uint64_t wv[kTabRpt][kTabWords];
#pragma unroll
    for (int i = 0; i < kTabRpt; ++i) {
      const int64_t r = rbase + (int64_t)i * kTabThreads + tid;
      const uint64_t* p = B + (row_first + (r < rows ? r : 0) * row_step) * stride + c * kTabWords;
#pragma unroll
      for (int q = 0; q < kTabWords; ++q) {
        const int64_t wd = c * kTabWords + q;
        uint64_t v = (r < rows && wd < Wc) ? p[q] : 0ull;
        if (wd == Wc - 1) v &= tail;
        wv[i][q] = v;
      }
    }
#pragma unroll
    for (int i = 0; i < kTabRpt; ++i) {
      double rowsum = 0.0;
#pragma unroll
      for (int q = 0; q < kTabWords; ++q) {
        const uint32_t lo = (uint32_t)wv[i][q], hi = (uint32_t)(wv[i][q] >> 32);
        const double* tq = tab + q * 8 * 256;
        const double t0 = tq[0 * 256 + (lo & 0xFF)];
        const double t1 = tq[1 * 256 + ((lo >> 8) & 0xFF)];
        const double t2 = tq[2 * 256 + ((lo >> 16) & 0xFF)];
        const double t3 = tq[3 * 256 + (lo >> 24)];
        const double t4 = tq[4 * 256 + (hi & 0xFF)];
        const double t5 = tq[5 * 256 + ((hi >> 8) & 0xFF)];
        const double t6 = tq[6 * 256 + ((hi >> 16) & 0xFF)];
        const double t7 = tq[7 * 256 + (hi >> 24)];
        rowsum += ((t0 + t1) + (t2 + t3)) + ((t4 + t5) + (t6 + t7));
      }
      acc[i] += rowsum;
    }
  }
#pragma unroll
  for (int i = 0; i < kTabRpt; ++i) {
    const int64_t r = rbase + (int64_t)i * kTabThreads + tid;
    if (r < rows) partial[(int64_t)blockIdx.y * rows + r] = acc[i];
  }
}

__global__ void tab_reduce_kernel(const double* partial, int64_t rows, int groups, const double* addend, double* out) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  // eight loads in flight; the partial sums are added in the order of their groups whatever the count is
  double s = addend ? addend[r] : 0.0;
  int g = 0;
  for (; g + 8 <= groups; g += 8) {
    double v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(g + u) * rows + r];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; g < groups; ++g) s += partial[(int64_t)g * rows + r];
  out[r] = s;
}

// ---- sparse rows: index lists ----------------------------------------------------------------
// idx[off[i] .. off[i+1]) = ascending columns of the set bits of row i; one wave per row
__global__ __launch_bounds__(kThreads) void rows_to_csr_kernel(const uint64_t* B, int64_t rows, int64_t cols, int64_t stride,
                                                               int64_t row_first, int64_t row_step, const int32_t* off,
                                                               int32_t* idx) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const int64_t Wc = (cols + 63) / 64;
  const uint64_t tail = (cols & 63) ? ((1ull << (cols & 63)) - 1ull) : ~0ull;
  for (int64_t i = wave; i < rows; i += nwaves) {
    const uint64_t* row = B + (row_first + i * row_step) * stride;
    int32_t base = off[i];
    for (int64_t w0 = 0; w0 < Wc; w0 += 64) {
      const int64_t wd = w0 + lane;
      uint64_t word = wd < Wc ? row[wd] : 0ull;
      if (wd == Wc - 1) word &= tail;
      const int cnt = __popcll(word);
      int pre = cnt;  // inclusive scan over the lanes
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(pre, o, 64);
        if (lane >= o) pre += v;
      }
      int32_t at = base + pre - cnt;
      while (word) {
        idx[at++] = (int32_t)(wd * 64 + __ffsll((long long)word) - 1);
        word &= word - 1;
      }
      base += __shfl(pre, 63, 64);
    }
  }
}

// out[i] = sum_{e in [off[i], off[i+1])} x[idx[e]]; one wave per row, rows taken from the long end first
__global__ __launch_bounds__(kThreads) void csr_gather_kernel(const int32_t* off, const int32_t* idx, int64_t rows,
                                                              const double* x, double* out) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t w = wave; w < rows; w += nwaves) {
    const int64_t i = rows - 1 - w;
    const int32_t a = off[i], b = off[i + 1];
    double s0 = 0.0, s1 = 0.0;
    int32_t e = a + lane;
    for (; e + 64 < b; e += 128) {
      s0 += x[idx[e]];
      s1 += x[idx[e + 64]];
    }
    if (e < b) s0 += x[idx[e]];
    double s = s0 + s1;
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) out[i] = s;
  }
}
}  // namespace

int ds_bit_spmv(ds_ctx* ctx, const uint64_t* B, int64_t rows, int64_t cols, int64_t stride, int64_t row_first,
                int64_t row_step, const double* x, double* out) {
  if (rows <= 0) return DS_OK;
  const int64_t rows_per_block = kSpmvRowsPerWave * (kThreads / 64);
  const int64_t blocks = (rows + rows_per_block - 1) / rows_per_block;
  if (blocks < (int64_t)ctx->num_cus) {
    hipLaunchKernelGGL(bit_spmv_rows_kernel, dim3((unsigned)((rows * 64 + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       ctx->stream, B, rows, cols, stride, row_first, row_step, x, out);
    DS_HIP(ctx, hipGetLastError());
    return DS_OK;
  }
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

size_t ds_bit_spmv_tab_ws_doubles(const ds_ctx* ctx, int64_t rows, int64_t cols) {
  const int64_t row_groups = (rows + kTabRows - 1) / kTabRows;
  const int64_t n_chunks = (cols + kTabCols - 1) / kTabCols;
  int64_t groups = (6 * (int64_t)ctx->num_cus + row_groups - 1) / (row_groups > 0 ? row_groups : 1);
  if (groups > n_chunks) groups = n_chunks;
  if (groups < 1) groups = 1;
  return (size_t)groups * (size_t)rows;
}

int ds_bit_spmv_tab(ds_ctx* ctx, const uint64_t* B, int64_t rows, int64_t cols, int64_t stride, int64_t row_first,
                    int64_t row_step, const double* x, const double* addend, double* out, double* ws,
                    hipEvent_t addend_ready) {
  if (rows <= 0) return DS_OK;
  const int64_t row_groups = (rows + kTabRows - 1) / kTabRows;
  const int64_t n_chunks = (cols + kTabCols - 1) / kTabCols;
  int64_t groups = (6 * (int64_t)ctx->num_cus + row_groups - 1) / row_groups;
  if (groups > n_chunks) groups = n_chunks;
  if (groups < 1) groups = 1;
  const int64_t cpg = (n_chunks + groups - 1) / groups;
  groups = (n_chunks + cpg - 1) / cpg;
  const size_t lds = (size_t)(kTabGroups * 256 + kTabGroups * 32 + kTabCols) * sizeof(double);
  DS_HIP(ctx, hipFuncSetAttribute((const void*)bit_spmv_tab_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  hipLaunchKernelGGL(bit_spmv_tab_kernel, dim3((unsigned)row_groups, (unsigned)groups), dim3(kTabThreads), lds, ctx->stream, B,
                     rows, cols, stride, row_first, row_step, x, ws, cpg, n_chunks);
  if (addend_ready) DS_HIP(ctx, hipStreamWaitEvent(ctx->stream, addend_ready, 0));  // the addend comes from another stream
  hipLaunchKernelGGL(tab_reduce_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, ctx->stream, ws, rows,
                     (int)groups, addend, out);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

int ds_rows_to_csr(ds_ctx* ctx, const uint64_t* B, int64_t rows, int64_t cols, int64_t stride, int64_t row_first,
                   int64_t row_step, const int32_t* off, int32_t* idx) {
  if (rows <= 0) return DS_OK;
  int64_t blocks = (rows * 64 + kThreads - 1) / kThreads;
  if (blocks > (int64_t)ctx->num_cus * 16) blocks = (int64_t)ctx->num_cus * 16;
  hipLaunchKernelGGL(rows_to_csr_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, ctx->stream, B, rows, cols, stride,
                     row_first, row_step, off, idx);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

int ds_csr_gather(ds_ctx* ctx, const int32_t* off, const int32_t* idx, int64_t rows, const double* x, double* out) {
  if (rows <= 0) return DS_OK;
  int64_t blocks = (rows * 64 + kThreads - 1) / kThreads;
  if (blocks > (int64_t)ctx->num_cus * 16) blocks = (int64_t)ctx->num_cus * 16;
  hipLaunchKernelGGL(csr_gather_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, ctx->stream, off, idx, rows, x, out);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}
