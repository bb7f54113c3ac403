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

// Transpose a bit matrix: in[rows x Win words] (row stride in_stride words, rows taken as row_first + i*row_step)
// -> out[cols x Wout words], Wout = ceil(rows/64); bit i of out row j = bit j of in row i.
// A workgroup of 512 threads takes a tile of 512 rows x 512 columns through LDS: every row is read in 64 contiguous
// bytes and every output row written in 64 contiguous bytes (one wave per 64x64 block with 8-byte accesses, the first
// version, left most of every cache line unused: 0.3 TB/s). Each wave transposes eight of the tile's 64x64 blocks in
// registers: lane = row, six rounds of swapping bit blocks with the lane 32, 16, ... 1 away.
constexpr int kTrThreads = 512;
constexpr int kTrPitch = 9;  // 64-bit words per LDS row of 8: lanes that read one word column of 64 rows spread over the banks

__device__ __forceinline__ uint64_t transpose64_in_wave(uint64_t x, int lane) {
  const uint64_t masks[6] = {0x00000000FFFFFFFFull, 0x0000FFFF0000FFFFull, 0x00FF00FF00FF00FFull,
                             0x0F0F0F0F0F0F0F0Full, 0x3333333333333333ull, 0x5555555555555555ull};
#pragma unroll
  for (int s = 0; s < 6; ++s) {
    const int j = 32 >> s;
    const uint64_t m = masks[s];
    const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)x, j, 64), hi = (uint32_t)__shfl_xor((int)(uint32_t)(x >> 32), j, 64);
    const uint64_t t = ((uint64_t)hi << 32) | lo;
    // rows whose index has bit j clear keep their low bit blocks and take the partner's low blocks as their high
    // ones; the others keep their high blocks and take the partner's high blocks as their low ones
    x = (lane & j) ? (((t >> j) & m) | (x & ~m)) : ((x & m) | ((t & m) << j));
  }
  return x;
}

__global__ __launch_bounds__(kTrThreads) void bit_transpose_kernel(const uint64_t* in, int64_t rows, int64_t cols,
                                                                   int64_t in_stride, int64_t row_first, int64_t row_step,
                                                                   uint64_t* out, int64_t Wout, int64_t tiles_c, int block_major) {
  __shared__ uint64_t tin[512 * kTrPitch];
  __shared__ uint64_t tout[512 * kTrPitch];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t Win = (cols + 63) / 64;
  const int64_t tr = blockIdx.x / tiles_c, tc = blockIdx.x % tiles_c;   // consecutive workgroups walk along a row block
  const int64_t r0 = tr * 512, w0 = tc * 8;
  // load: 8 lanes per row (64 contiguous bytes), 64 rows per step
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int r = k * 64 + (t >> 3), w = t & 7;
    uint64_t v = 0;
    if (r0 + r < rows && w0 + w < Win) v = in[(row_first + (r0 + r) * row_step) * in_stride + w0 + w];
    tin[r * kTrPitch + w] = v;
  }
  __syncthreads();
  // wave `wave` transposes the blocks (row block rbi, word column wave) for the eight row blocks
#pragma unroll
  for (int rbi = 0; rbi < 8; ++rbi) {
    const uint64_t x = transpose64_in_wave(tin[(rbi * 64 + lane) * kTrPitch + wave], lane);
    tout[(wave * 64 + lane) * kTrPitch + rbi] = x;   // lane = column within the word column, word = row block
  }
  __syncthreads();
  if (block_major) {
    // out[row block][column] (Win * 64 columns per row block): a wave writes the 64 columns of one row block, 512
    // contiguous bytes
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int c = k * 64 + lane, w = wave;
      const int64_t col = w0 * 64 + c, ow = tr * 8 + w;
      if (col < Win * 64 && ow < Wout) out[ow * (Win * 64) + col] = tout[c * kTrPitch + w];
    }
    return;
  }
  // store: 8 lanes per output row (64 contiguous bytes)
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int c = k * 64 + (t >> 3), w = t & 7;
    const int64_t col = w0 * 64 + c, ow = tr * 8 + w;
    if (col < cols && ow < Wout) out[col * Wout + ow] = tout[c * kTrPitch + w];
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

// ---- dense rows: product on the int8 matrix cores ------------------------------------------
// out[i] = sum over set bits j of row i of x[j], for rows dense enough that one look-up or one
// gather per set bit (or per byte of mask) costs more than streaming the bits. The product is a
// (rows x cols 0/1 matrix) . (cols x 7 matrix of base-256 digits of x): exact integer arithmetic.
//  * x is scaled by a power of two so that max|x| < 2^54 and rounded to integers (the same 2^-54
//    relative step for every entry); each integer is written in seven balanced base-256 digits
//    (-128..127), one int8 plane per digit (`quantize_kernel`).
//  * A operand of v_mfma_i32_16x16x64_i8 = 16 rows x 64 columns of mask bits as bytes. A lane holds
//    16 bytes of one row; the bytes come from the lane's four 32-bit mask words by ONE AND each:
//    word & (0x01010101 << j) puts bit j of every mask byte into a byte of its own (value 2^j), so
//    operand j multiplies the columns {8i + j} and its accumulator carries the factor 2^(j & 3)
//    (bits 4..7 after a shift of the word by 4), divided out exactly at the end. The digit planes
//    are stored permuted to match: within every 128 columns, position j<<4 | v<<2 | i holds column
//    v<<5 | i<<3 | j, so the B operand of (word group, j) is 16 contiguous bytes.
//  * B operand = digits (7 of the 16 columns used; the eighth plane is zero and serves the idle
//    columns). The planes of a 1024-column chunk are staged in LDS once per workgroup and read by
//    all of its waves, one (half, nibble) group of four operands ahead of their use.
//  * A wave owns 64 rows (four 16-row tiles); per chunk every row is visited with 128 contiguous
//    bytes (two 16-byte loads per lane and tile), requested one chunk ahead.
// The per-column-group partial sums are int32 (exact) and are added up, recombined
// (sum_d 256^d S_d, as two exact integer halves) and rescaled by a second kernel, so the result does not
// depend on the grouping.
typedef int v4i __attribute__((ext_vector_type(4)));
constexpr int kMmTiles = 4;                          // 16-row tiles per wave
constexpr int kMmWaves = 4;                          // waves per workgroup
constexpr int kMmWaveRows = 16 * kMmTiles;
constexpr int kMmRows = kMmWaveRows * kMmWaves;      // rows per workgroup
constexpr int kMmChunk = 1024;                       // columns per step
constexpr int kMmHalves = kMmChunk / 512;            // 64-byte pieces of a row per chunk
constexpr int kMmDigits = 7;
constexpr int kMmPlanes = 8;
constexpr int kMmPlanePitch = kMmChunk + 16;         // LDS pitch of a plane: the eight planes start 16 bytes (4 banks) apart
constexpr int64_t kMmMaxGroupCols = 1 << 20;         // 2^20 columns * 128 * 2^3 = 2^30: the int32 accumulators cannot overflow

// slot: bit pattern of max |x| over the call (0 on entry; non-negative doubles order like their bit patterns)
__global__ __launch_bounds__(256) void absmax_kernel(const double* x, int64_t n, unsigned long long* slot) {
  unsigned long long m = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(x[i]) & 0x7fffffffffffffffull;
    m = b > m ? b : m;
  }
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long t = __shfl_xor(m, o, 64);
    m = t > m ? t : m;
  }
  if ((threadIdx.x & 63) == 0 && m) atomicMax(slot, m);
}

// The fixed-point form of a vector: scal[0] = the power of two that turns integer results back into the scale of x
// (NaN if the vector holds a non-finite value: the products are then NaN everywhere). Two roles per thread:
//  * digit planes of xp[0..n) (npad > 0): one thread per 4 plane positions (i = 0..3: columns 8 apart);
//  * q64[i] = round(xq[i] * 2^f) for i < qlen (the index-tile products read these): four entries per thread.
__global__ __launch_bounds__(256) void quantize_kernel(const double* xp, int64_t n, int64_t npad, const unsigned long long* slot,
                                                       int8_t* D, double* scal, const double* xq, int64_t qlen, long long* q64) {
  const double mx = __longlong_as_double((long long)*slot);
  const bool finite = mx < __longlong_as_double(0x7ff0000000000000ll);
  int e = 0;
  if (finite && mx > 0.0) frexp(mx, &e);   // mx < 2^e
  const int f = 54 - e;
  const int64_t q4 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q4 == 0) scal[0] = finite ? ldexp(1.0, -f) : __longlong_as_double(0x7ff8000000000000ll);
  const int64_t pos0 = q4 * 4;
  if (pos0 < qlen) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (pos0 + i < qlen) q64[pos0 + i] = finite ? __double2ll_rn(ldexp(xq[pos0 + i], f)) : 0ll;
  }
  if (pos0 >= npad) return;
  const int p = (int)(pos0 & 127);
  const int j = p >> 4, v = (p >> 2) & 3;
  const int64_t colbase = (pos0 & ~(int64_t)127) + (v << 5 | j);
  int32_t packed[kMmDigits] = {0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t col = colbase + (i << 3);
    long long q = (finite && col < n) ? __double2ll_rn(ldexp(xp[col], f)) : 0ll;
#pragma unroll
    for (int d = 0; d < kMmDigits; ++d) {
      const int di = (int)(int8_t)(q & 0xFF);
      q = (q - di) >> 8;
      packed[d] |= (di & 0xFF) << (8 * i);
    }
  }
#pragma unroll
  for (int d = 0; d < kMmDigits; ++d) *(int32_t*)(D + d * npad + pos0) = packed[d];
}

__global__ __launch_bounds__(kMmWaves * 64) void bit_spmv_mm_kernel(const uint64_t* B, int64_t rows, int64_t cols, int64_t stride,
                                                                    int64_t row_first, int64_t row_step, const int8_t* D,
                                                                    int64_t dstride, int32_t* partial, int64_t chunks_per_group,
                                                                    int64_t n_chunks) {
  __shared__ __align__(16) int8_t Bs[2][kMmPlanes * kMmPlanePitch];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, g = lane >> 4;
  const int64_t Wc = (cols + 63) / 64;
  const int64_t wave_row0 = ((int64_t)blockIdx.x * kMmWaves + wave) * kMmWaveRows;
  const int64_t c_begin = (int64_t)blockIdx.y * chunks_per_group;
  const int64_t c_end = c_begin + chunks_per_group < n_chunks ? c_begin + chunks_per_group : n_chunks;
  const int64_t row_bytes = row_step * stride * 8;
  const char* Bb = (const char*)(B + row_first * stride);
  const uint32_t lane_off = (uint32_t)r16 * (uint32_t)row_bytes;   // the host keeps 16 * row_bytes below 2^32
  v4i acc[kMmTiles][4];
#pragma unroll
  for (int t = 0; t < kMmTiles; ++t)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[t][q] = v4i{0, 0, 0, 0};
  uint32_t a_cur[kMmTiles][4 * kMmHalves], a_next[kMmTiles][4 * kMmHalves];
  // Rows past the end are read from a live row and never stored; in the last chunk, words past the row's end are
  // read from its last word and meet zero digits (the planes are zero from column `cols` on).
  // (one 16-byte load per lane, tile and half: as two 8-byte loads the same bytes took twice the requests and the
  // kernel ran 17 % slower)
  typedef uint32_t u4a8 __attribute__((ext_vector_type(4), aligned(8)));   // rows are 8-byte aligned
  auto load_a = [&](uint32_t (&a)[kMmTiles][4 * kMmHalves], int64_t c) {
    if (c != n_chunks - 1) {
#pragma unroll
      for (int t = 0; t < kMmTiles; ++t) {
        const int64_t r_t = wave_row0 + 16 * t;
        const char* base = Bb + (r_t < rows ? r_t : rows - 1) * row_bytes;   // uniform over the wave
        const uint32_t lo = (r_t + r16 < rows ? lane_off : 0u) + (uint32_t)(c * (kMmChunk / 8) + g * 16);
#pragma unroll
        for (int h = 0; h < kMmHalves; ++h) {
          const u4a8 v = *(const u4a8*)(base + (lo + h * 64));
          a[t][4 * h + 0] = v.x;
          a[t][4 * h + 1] = v.y;
          a[t][4 * h + 2] = v.z;
          a[t][4 * h + 3] = v.w;
        }
      }
    } else {
#pragma unroll
      for (int t = 0; t < kMmTiles; ++t) {
        const int64_t r_t = wave_row0 + 16 * t;
        const char* base = Bb + (r_t < rows ? r_t : rows - 1) * row_bytes;
        const uint32_t lo = r_t + r16 < rows ? lane_off : 0u;
#pragma unroll
        for (int h = 0; h < kMmHalves; ++h) {
          const int64_t w0 = c * (kMmChunk / 64) + h * 8 + g * 2, w1 = w0 + 1;
          const uint32_t cb0 = (uint32_t)(w0 < Wc ? w0 : Wc - 1) * 8u, cb1 = (uint32_t)(w1 < Wc ? w1 : Wc - 1) * 8u;
          const uint64_t v0 = *(const uint64_t*)(base + (lo + cb0)), v1 = *(const uint64_t*)(base + (lo + cb1));
          a[t][4 * h + 0] = (uint32_t)v0;
          a[t][4 * h + 1] = (uint32_t)(v0 >> 32);
          a[t][4 * h + 2] = (uint32_t)v1;
          a[t][4 * h + 3] = (uint32_t)(v1 >> 32);
        }
      }
    }
  };
  // staging of a chunk's digit planes: thread -> (plane, 32-byte segment)
  static_assert(kMmWaves * 64 * 32 == kMmPlanes * kMmChunk, "one 32-byte segment per thread");
  const int st_plane = tid / (kMmChunk / 32), st_seg = tid % (kMmChunk / 32);
  const int8_t* st_src = D + (int64_t)st_plane * dstride + st_seg * 32;
  const int st_dst = st_plane * kMmPlanePitch + st_seg * 32;
  v4i s0, s1;
  auto stage_load = [&](int64_t c) {
    s0 = *(const v4i*)(st_src + c * kMmChunk);
    s1 = *(const v4i*)(st_src + c * kMmChunk + 16);
  };
  auto stage_store = [&](int buf) {
    *(v4i*)(&Bs[buf][st_dst]) = s0;
    *(v4i*)(&Bs[buf][st_dst + 16]) = s1;
  };
  const int b_off = (r16 < kMmDigits ? r16 : kMmDigits) * kMmPlanePitch + g * 128;   // plane 7 is all zero
  stage_load(c_begin);
  load_a(a_cur, c_begin);
  stage_store(0);
  __syncthreads();
  int buf = 0;
  for (int64_t c = c_begin; c < c_end; ++c) {
    const int64_t cn = c + 1 < c_end ? c + 1 : c;   // (the last chunk is requested again and not used)
    stage_load(cn);
    load_a(a_next, cn);
    const int8_t* bs = &Bs[buf][b_off];
    v4i bq[2][4];
#pragma unroll
    for (int q = 0; q < 4; ++q) bq[0][q] = *(const v4i*)(bs + q * 16);
#pragma unroll
    for (int gi = 0; gi < 2 * kMmHalves; ++gi) {
      const int h = gi >> 1, hi = gi & 1;
      if (gi + 1 < 2 * kMmHalves) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          bq[(gi + 1) & 1][q] = *(const v4i*)(bs + ((gi + 1) >> 1) * 512 + (4 * ((gi + 1) & 1) + q) * 16);
      }
#pragma unroll
      for (int t = 0; t < kMmTiles; ++t) {
        uint32_t x0 = a_cur[t][4 * h + 0], x1 = a_cur[t][4 * h + 1], x2 = a_cur[t][4 * h + 2], x3 = a_cur[t][4 * h + 3];
        if (hi) {
          x0 >>= 4;
          x1 >>= 4;
          x2 >>= 4;
          x3 >>= 4;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const uint32_t m = 0x01010101u << q;
          const v4i av = {(int)(x0 & m), (int)(x1 & m), (int)(x2 & m), (int)(x3 & m)};
          acc[t][q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bq[gi & 1][q], acc[t][q], 0, 0, 0);
        }
      }
    }
    stage_store(buf ^ 1);
    __syncthreads();   // every wave is done with Bs[buf]; Bs[buf ^ 1] is complete
    buf ^= 1;
#pragma unroll
    for (int t = 0; t < kMmTiles; ++t)
#pragma unroll
      for (int k = 0; k < 4 * kMmHalves; ++k) a_cur[t][k] = a_next[t][k];
  }
  // lane (digit r16, lane group g) holds rows 4g + v of every tile
  if (r16 < kMmPlanes) {
#pragma unroll
    for (int t = 0; t < kMmTiles; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int64_t row = wave_row0 + 16 * t + 4 * g + v;
        if (row < rows)
          partial[((int64_t)blockIdx.y * rows + row) * kMmPlanes + r16] =
              acc[t][0][v] + (acc[t][1][v] >> 1) + (acc[t][2][v] >> 2) + (acc[t][3][v] >> 3);
      }
  }
}

// out[r] = (addend[r] or 0) + scal[0] * sum_d 256^d * (sum over the column groups of digit sum d); clears the
// maximum slot for the next product if asked to
__global__ __launch_bounds__(256) void mm_reduce_kernel(const int32_t* partial, int64_t rows, int groups, const double* scal,
                                                        const double* addend, double* out, unsigned long long* slot) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r == 0 && slot) *slot = 0ull;
  if (r >= rows) return;
  const double val = ds_mm_sum(partial, rows, groups, r) * scal[0];
  out[r] = addend ? addend[r] + val : val;
}

// ---- sparse rows: index lists (the input of the tile build) ------------------------------------
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
  const int64_t tiles_r = (rows + 511) / 512, tiles_c = (Win + 7) / 8;
  if (tiles_r < 1 || tiles_c < 1) return DS_OK;
  if (tiles_r * tiles_c > 0x7fffffffLL) return ds_fail(ctx, DS_EINVAL, "bit matrix too large to transpose");
  hipLaunchKernelGGL(bit_transpose_kernel, dim3((unsigned)(tiles_r * tiles_c)), dim3(kTrThreads), 0, ctx->stream, in, rows, cols,
                     in_stride, row_first, row_step, out, Wout, tiles_c, 0);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

int ds_bit_transpose_blocks(ds_ctx* ctx, const uint64_t* in, int64_t rows, int64_t cols, int64_t in_stride, int64_t row_step,
                            uint64_t* out) {
  const int64_t Wout = (rows + 63) / 64, Win = (cols + 63) / 64;
  const int64_t tiles_r = (rows + 511) / 512, tiles_c = (Win + 7) / 8;
  if (tiles_r < 1 || tiles_c < 1) return DS_OK;
  if (tiles_r * tiles_c > 0x7fffffffLL) return ds_fail(ctx, DS_EINVAL, "bit matrix too large to transpose");
  hipLaunchKernelGGL(bit_transpose_kernel, dim3((unsigned)(tiles_r * tiles_c)), dim3(kTrThreads), 0, ctx->stream, in, rows, cols,
                     in_stride, (int64_t)0, row_step, out, Wout, tiles_c, 1);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

static void mm_shape(const ds_ctx* ctx, int64_t rows, int64_t cols, ds_mm_plan* p) {
  p->rows = rows;
  p->cols = cols;
  p->row_groups = (rows + kMmRows - 1) / kMmRows;
  p->n_chunks = (cols + kMmChunk - 1) / kMmChunk;
  p->npad = p->n_chunks * kMmChunk;
  // Column groups: two workgroups fit a compute unit (registers), so the launch runs in rounds of 2 x CUs workgroups;
  // among the splits that give 3 to 10 rounds, take the one that wastes least of its last round and of its last
  // group's chunk range (config 4's forward product: 9 groups = 3.97 rounds instead of 10 = 4.41).
  const int64_t cap = 2 * (int64_t)ctx->num_cus, rg = p->row_groups > 0 ? p->row_groups : 1;
  const int64_t max_cpg = kMmMaxGroupCols / kMmChunk;
  int64_t g_lo = (3 * cap + rg - 1) / rg, g_hi = (10 * cap + rg - 1) / rg;
  if (g_lo < 1) g_lo = 1;
  if (g_hi > p->n_chunks) g_hi = p->n_chunks;
  if (g_lo > g_hi) g_lo = g_hi;
  if (g_lo < 1) g_lo = g_hi = 1;
  double best = -1.0;
  p->cpg = p->n_chunks > 0 ? p->n_chunks : 1;
  p->groups = 1;
  for (int64_t g = g_lo; g <= g_hi; ++g) {
    int64_t cpg = (p->n_chunks + g - 1) / g;
    if (cpg > max_cpg) cpg = max_cpg;
    if (cpg < 1) cpg = 1;
    const int64_t groups = (p->n_chunks + cpg - 1) / cpg;
    const int64_t wgs = rg * groups, rounds = (wgs + cap - 1) / cap;
    const double eff = (double)wgs / (double)(rounds * cap) * (double)p->n_chunks / (double)(groups * cpg);
    if (eff > best + 1e-9) {
      best = eff;
      p->cpg = cpg;
      p->groups = groups;
    }
  }
}

size_t ds_bit_spmv_mm_ws_bytes(const ds_ctx* ctx, int64_t rows, int64_t cols) {
  ds_mm_plan p;
  mm_shape(ctx, rows, cols, &p);
  return ds_align((size_t)kMmPlanes * p.npad) + ds_align((size_t)p.groups * rows * kMmPlanes * 4);
}

int ds_bit_spmv_mm_prepare(ds_ctx* ctx, int64_t rows, int64_t cols, void* ws, ds_mm_plan* plan) {
  mm_shape(ctx, rows, cols, plan);
  char* p = (char*)ws;
  plan->D = (int8_t*)p;
  plan->partial = (int32_t*)(p + ds_align((size_t)kMmPlanes * plan->npad));
  DS_HIP(ctx, hipMemsetAsync(plan->D + (size_t)kMmDigits * plan->npad, 0, plan->npad, ctx->stream));  // the zero plane
  return DS_OK;
}

int ds_vec_quantize(ds_ctx* ctx, const double* x_all, int64_t len_all, const ds_mm_plan* planes, const double* x_planes,
                    const double* x_q, int64_t qlen, long long* q64, double* scal, int with_absmax) {
  unsigned long long* slot = (unsigned long long*)(scal + 1);
  int64_t mb = (len_all + 2047) / 2048;
  if (mb > 2 * (int64_t)ctx->num_cus) mb = 2 * (int64_t)ctx->num_cus;
  if (mb < 1) mb = 1;
  if (with_absmax) hipLaunchKernelGGL(absmax_kernel, dim3((unsigned)mb), dim3(256), 0, ctx->stream, x_all, len_all, slot);
  const bool with_planes = planes && planes->rows > 0;
  const int64_t npad = with_planes ? planes->npad : 0;
  const int64_t span = npad > qlen ? npad : qlen;
  hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)((span / 4 + 256) / 256)), dim3(256), 0, ctx->stream, x_planes,
                     with_planes ? planes->cols : 0, npad, slot, with_planes ? planes->D : nullptr, scal, x_q, qlen, q64);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

int ds_bit_spmv_mm_product(ds_ctx* ctx, const ds_mm_plan* p, const uint64_t* B, int64_t stride, int64_t row_first,
                           int64_t row_step, const double* scal, const double* addend, double* out, int clear_slot) {
  if (p->rows <= 0) return DS_OK;
  if (row_step * stride * 8 * 16 >= ((int64_t)1 << 32))
    return ds_fail(ctx, DS_EINTERNAL, "matrix-core product: rows of %lld bytes are too far apart", (long long)(row_step * stride * 8));
  hipLaunchKernelGGL(bit_spmv_mm_kernel, dim3((unsigned)p->row_groups, (unsigned)p->groups), dim3(kMmWaves * 64), 0, ctx->stream,
                     B, p->rows, p->cols, stride, row_first, row_step, p->D, p->npad, p->partial, p->cpg, p->n_chunks);
  if (out)
    hipLaunchKernelGGL(mm_reduce_kernel, dim3((unsigned)((p->rows + 255) / 256)), dim3(256), 0, ctx->stream, p->partial, p->rows,
                       (int)p->groups, scal, addend, out, clear_slot ? (unsigned long long*)(scal + 1) : (unsigned long long*)nullptr);
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
