// Direct solve of the Kernel-SHAP regression for small player counts:
// popcount Gram matrix + blocked Cholesky, all accumulation in fp64.
//
// Paper, "Distributed Shapley Computations": the direct method forms
// G = M^T W M and r = M^T W y and solves G phi = r. Here the efficiency
// decomposition (f(N) = phi_0 + sum phi_i) is imposed exactly: with
// delta = y_1 - y_0, psi = phi - delta/n, P = I - 11^T/n and
// t_i = y_i - y_0 - (delta/n)|S_i|, psi solves (P G P + gamma 11^T/n) psi = P c,
// c = M^T W t, and any gamma > 0 leaves psi orthogonal to 1.
//
// G[a][b] = sum_i w_i z_ia z_ib is computed from the transposed bit matrix: a
// 64-row word whose rows share one weight contributes w * popcount(col_a & col_b);
// a word that straddles weight classes is a dense 64-row contraction on the matrix cores.
#include <stdlib.h>

#include "internal.h"
#include "solve_common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kTile = 64;
constexpr int kChunk = 32;  // 64-row words per LDS chunk

// which rows enter the sums, with which weight and right-hand-side coefficient.
// Paired rows (2r, 2r+1 complementary, one weight w): z z^T + zc zc^T = 2 z z^T - z 1^T - 1 z^T + 11^T and
// t z + tc zc = (t - tc) z + tc 1; the terms with 1 vanish under the projection P, so only the small
// member is used, with weight 2w and coefficient w (t_2r - t_2r+1). Otherwise every row is used.
__global__ void used_row_weights_kernel(const float* w, int64_t R, int paired, float* gw) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= R) return;
  const int64_t i = paired ? 2 * r : r;
  const float wi = i < 2 ? 0.f : w[i];  // the two constraint rows carry no weight
  gw[r] = paired ? 2.0f * wi : wi;
}

__global__ void used_row_rhs_kernel(const float* wc, const double* t, int64_t R, int paired, double* gc) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= R) return;
  gc[r] = paired ? (double)wc[2 * r] * (t[2 * r] - t[2 * r + 1]) : (double)wc[r] * t[r];
}

// per word of 64 rows: the common weight and how the Gram kernel treats the word:
// 1 = one weight (popcount), 0 = mixed weights and sparse rows (walk the set bits of the AND),
// 2 = mixed weights and dense rows (matrix cores). The density is read off the first row of the word
// (rows are ordered by size): with a fraction p of the columns set, a pair of columns shares about 64 p^2
// rows of the word, and walking them costs more than the fixed-price contraction from p of about 0.08 on (measured).
constexpr float kDenseFraction = 0.08f;
__global__ void word_weights_kernel(const float* w, int64_t k, int64_t KW, const uint64_t* Z, int64_t W, int64_t n,
                                    int64_t row_step, float dense_fraction, const uint64_t* keep, float* wu,
                                    int32_t* uni) {
  const int64_t wd = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (wd >= KW) return;
  const int64_t i0 = wd * 64;
  const uint64_t km = keep[wd];  // rows of this word that are left to the column-wise kernel
  if (km == 0ull) {
    wu[wd] = 0.f;
    uni[wd] = 3;  // nothing to do
    return;
  }
  const int fb = __ffsll((long long)km) - 1;
  const float first = w[i0 + fb];
  int same = 1;
  for (int b = fb + 1; b < 64; ++b) {
    const int64_t i = i0 + b;
    if (((km >> b) & 1ull) && i < k && w[i] != first) same = 0;
  }
  wu[wd] = first;
  int mode = same;
  if (!same) {
    const uint64_t* zr = Z + (i0 + fb) * row_step * W;
    int64_t c = 0;
    for (int64_t x = 0; x < W; ++x) c += __popcll(zr[x]);
    if ((float)c > dense_fraction * (float)n) mode = 2;
  }
  uni[wd] = mode;
}

// ---- sparse rows: row-wise outer products -------------------------------------------------------
// A row with s of n columns set touches s^2 entries of G, while the column-wise kernel pays for all
// n^2/2 pairs of columns whatever the row holds; up to a density of about a tenth the row-wise form is the
// cheaper one, and in a Kernel-SHAP sample most rows are far sparser than that. Rows are split by their
// own popcount: sparse ones go to gram_rows_kernel, the others stay with the column-wise kernel
// (`keep` holds their bits per 64-row word).
//   Zc[cb][r] = word cb of row r (zero for a kept row): the 64 columns of a tile side for all rows, contiguous.
//   wq[r]     = weight of row r in fixed point, w_r * 2^e with e chosen so that the sum of all weights stays
//               below 2^62: every entry of G is a sum over a subset of the rows, so the integer sums cannot
//               overflow, they are exact, and they do not depend on the order of the atomic additions.
constexpr int kSparseDivisor = 12;  // rows with at most n / 12 columns set are sparse (measured optimum: flat from 8 to 16)

// scale[0] = 2^e (0 if the weights are not all finite and non-negative: then every row is kept)
__global__ __launch_bounds__(kThreads) void gram_scale_kernel(const float* gw, int64_t R, double* scale) {
  __shared__ double sh[kThreads];
  __shared__ int bad[kThreads];
  double a = 0.0;
  int b = 0;
  for (int64_t i = threadIdx.x; i < R; i += kThreads) {
    const float v = gw[i];
    if (!(v >= 0.f) || v > 3.0e38f) b = 1;
    a += (double)v;
  }
  sh[threadIdx.x] = a;
  bad[threadIdx.x] = b;
  __syncthreads();
  if (threadIdx.x == 0) {
    double x = 0.0;
    int anyb = 0;
    for (int i = 0; i < kThreads; ++i) {
      x += sh[i];
      anyb |= bad[i];
    }
    double sc = 0.0;
    if (!anyb && x > 0.0 && x < 1e300) {
      int e;
      frexp(x, &e);  // x < 2^e
      sc = ldexp(1.0, 61 - e);
    }
    scale[0] = sc;
  }
}

// one wave per used row
__global__ __launch_bounds__(kThreads) void gram_row_class_kernel(const uint64_t* Z, int64_t R, int64_t W, int64_t n,
                                                                  int64_t row_step, const float* gw, const double* scale,
                                                                  int sparse_divisor, uint64_t* Zc,
                                                                  unsigned long long* keep, unsigned long long* wq) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const double sc = scale[0];
  for (int64_t r = wave; r < R; r += nwaves) {
    const uint64_t* zr = Z + r * row_step * W;
    int c = 0;
    for (int64_t x = lane; x < W; x += 64) c += __popcll(zr[x]);
    for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
    const bool sparse = sc > 0.0 && (int64_t)c * sparse_divisor <= n;
    for (int64_t x = lane; x < W; x += 64) Zc[x * R + r] = sparse ? zr[x] : 0ull;
    if (lane == 0) {
      wq[r] = sparse ? (unsigned long long)llrint((double)gw[r] * sc) : 0ull;
      if (!sparse) atomicOr(&keep[r >> 6], 1ull << (r & 63));
    }
  }
}

// One 64x64 tile of G per workgroup (lower tiles); streams the two column-block words of every row.
__global__ __launch_bounds__(kThreads) void gram_rows_kernel(const uint64_t* Zc, const unsigned long long* wq, int64_t R,
                                                             int64_t n, const double* scale, double* G) {
  const int ta = blockIdx.y, tb = blockIdx.x;
  if (tb > ta) return;
  __shared__ unsigned long long acc[kTile * kTile];
  const int tid = threadIdx.x;
  for (int i = tid; i < kTile * kTile; i += kThreads) acc[i] = 0ull;
  __syncthreads();
  const uint64_t* Ac = Zc + (size_t)ta * R;
  const uint64_t* Bc = Zc + (size_t)tb * R;
  constexpr int kRowsPerStep = 8;  // rows per step: their loads are in flight together (addresses clamped, not skipped)
  for (int64_t r0 = tid; r0 < R; r0 += kRowsPerStep * kThreads) {
    uint64_t av[kRowsPerStep], bv[kRowsPerStep];
    unsigned long long wvv[kRowsPerStep];
#pragma unroll
    for (int u = 0; u < kRowsPerStep; ++u) {
      const int64_t r = r0 + (int64_t)u * kThreads, rc = r < R ? r : R - 1;
      av[u] = Ac[rc];
      bv[u] = Bc[rc];
      wvv[u] = wq[rc];
    }
#pragma unroll
    for (int u = 0; u < kRowsPerStep; ++u) {
      if (r0 + (int64_t)u * kThreads >= R || av[u] == 0ull || bv[u] == 0ull) continue;
      const unsigned long long wv = wvv[u];
      uint64_t am = av[u];
      while (am) {
        const int a = __ffsll((long long)am) - 1;
        am &= am - 1;
        uint64_t bm = bv[u];
        while (bm) {
          const int b = __ffsll((long long)bm) - 1;
          bm &= bm - 1;
          atomicAdd(&acc[a * kTile + b], wv);
        }
      }
    }
  }
  __syncthreads();
  const double sc = scale[0];
  const double inv = sc > 0.0 ? 1.0 / sc : 0.0;
  for (int i = tid; i < kTile * kTile; i += kThreads) {
    const int64_t a = (int64_t)ta * kTile + (i >> 6), b = (int64_t)tb * kTile + (i & 63);
    if (a < n && b < n) {
      const double v = (double)acc[i] * inv;
      G[a * n + b] = v;
      if (ta != tb) G[b * n + a] = v;
    }
  }
}

// One 64x64 tile of G per workgroup and slice of the row words (split-K); each slice
// writes its own full symmetric partial matrix, summed later in a fixed order.
// A word of 64 rows that share one weight costs an AND and a popcount per pair of columns. A word that
// straddles weight classes (most words past the first few classes: a class soon has fewer than 64 rows)
// either walks the set bits of the AND (sparse rows) or, when its rows are dense, is treated as the small
// dense contraction it is, sum_r (w_r z_ra) z_rb, on the matrix cores. The fp32 weight is split into three
// bfloat16 pieces (w = w1 + w2 + w3 to 24 bits; a bit is exactly 0 or 1 in bfloat16), so the contraction runs
// as three v_mfma_f32_32x32x8bf16_1k per 8 rows with fp32 accumulation, several times the rate of the fp32
// instruction: lane l supplies A[m = l%32][k = 4*(l/32) + j] = piece of row r * bit r of column m's word and
// B[k][n = l%32] = bit r of column n's word, r = 8 kb + k, j < 4 (two values per register). Operands are
// made with look-ups: a 16-entry LDS table turns four bits into the two registers of 16-bit masks (or of
// bfloat16 ones for B), which the packed weight pieces are ANDed with. Each wave owns a 32x32 quadrant of the
// tile (accumulator register i of lane l is D[8*(i/4) + 4*(l/32) + i%4][l%32]). Both paths add up in fp32
// within a chunk of 32 words and in fp64 across chunks.
typedef float gram_f16_t __attribute__((ext_vector_type(16)));
typedef short gram_s4_t __attribute__((ext_vector_type(4)));
typedef unsigned int gram_u2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t bf16_bits_rn(float x) {  // nearest-even bfloat16 of a finite float, as 16 bits
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
// 16-bit lane masks of two bits: bit 0 -> low half, bit 1 -> high half
__device__ __forceinline__ uint32_t pair_mask(uint32_t two_bits) {
  return ((0u - (two_bits & 1u)) & 0xFFFFu) | ((0u - ((two_bits >> 1) & 1u)) & 0xFFFF0000u);
}

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 4))) void gram_kernel(const uint64_t* Zt, int64_t n, int64_t k, int64_t KW,
                                                        const float* w, const float* wu, const int32_t* uni,
                                                        const uint64_t* keep, double* Gp, int64_t words_per_slice) {
  const int ta = blockIdx.y, tb = blockIdx.x;
  if (tb > ta) return;
  // As | Bs during the accumulation; reused as one 64 x 65 fp64 tile when the two paths are merged
  __shared__ __attribute__((aligned(16))) uint64_t raw[2 * kTile * (kChunk + 1)];
  static_assert(sizeof(uint64_t) * 2 * kTile * (kChunk + 1) >= sizeof(double) * kTile * (kTile + 1), "merge tile must fit");
  uint64_t (*As)[kChunk + 1] = (uint64_t (*)[kChunk + 1])raw;
  uint64_t (*Bs)[kChunk + 1] = (uint64_t (*)[kChunk + 1])(raw + kTile * (kChunk + 1));
  __shared__ float wrow[kChunk * 64];
  __shared__ gram_u2_t wpk[3][kChunk * 16];  // weight pieces as bfloat16, rows 4j..4j+3 of a word per entry
  __shared__ gram_u2_t tabA[16], tabB[16];   // four bits -> 16-bit masks / bfloat16 ones (two registers)
  __shared__ float wus[kChunk];
  __shared__ int unis[kChunk];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
  if (tid < 16) {
    const gram_u2_t m = {pair_mask(tid & 3u), pair_mask((uint32_t)tid >> 2)};
    tabA[tid] = m;
    tabB[tid] = gram_u2_t{m.x & 0x3F803F80u, m.y & 0x3F803F80u};
  }
  const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;
  const int64_t a0 = (int64_t)ta * kTile, b0 = (int64_t)tb * kTile;
  double* G = Gp + (size_t)blockIdx.z * n * n;
  const int64_t wbeg = (int64_t)blockIdx.z * words_per_slice;
  const int64_t wend = wbeg + words_per_slice < KW ? wbeg + words_per_slice : KW;
  double acc[4][4];   // popcount path: elements (ty + 16 i, tx + 16 j)
  double accm[16];    // matrix-core path: elements (wi + 8*(i/4) + 4*half + i%4, wj + l32)
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      acc[i][j] = 0.0;
      accm[4 * i + j] = 0.0;
    }
  for (int64_t wd0 = wbeg; wd0 < wend; wd0 += kChunk) {
    {  // a chunk none of whose rows is kept (all sparse: done by the row-wise kernel) is not even loaded
      const int64_t wd = wd0 + (tid & (kChunk - 1));
      const bool any = wd < wend && keep[wd] != 0ull;
      if (!__syncthreads_or(any)) continue;
    }
    // Everything the chunk needs from global memory is fetched into registers first (addresses clamped instead of
    // skipped) and only then stored to LDS: a loop that loads and stores element by element pays one memory latency
    // per element, about twenty per chunk.
    {
      constexpr int kZ = kTile * kChunk / kThreads;  // mask words per thread and operand
      constexpr int kWr = kChunk * 64 / kThreads;    // row weights per thread
      constexpr int kWp = kChunk * 16 / kThreads;    // groups of four rows per thread
      static_assert(kThreads % kChunk == 0, "a thread stays in one word column of the chunk");
      uint64_t za[kZ], zb[kZ];
      float wr_[kWr], w4[kWp][4];
      const int cz = tid % kChunk;  // this thread's word of the chunk (the same for all its elements)
      const int64_t wdz = wd0 + cz < wend ? wd0 + cz : wend - 1;
      const uint64_t kp = keep[wdz];
#pragma unroll
      for (int u = 0; u < kZ; ++u) {
        const int r = (tid + u * kThreads) / kChunk;
        const int64_t ra = a0 + r < n ? a0 + r : n - 1, rb = b0 + r < n ? b0 + r : n - 1;
        za[u] = Zt[ra * KW + wdz];
        zb[u] = Zt[rb * KW + wdz];
      }
#pragma unroll
      for (int u = 0; u < kWr; ++u) {
        const int64_t i = wd0 * 64 + tid + u * kThreads;
        wr_[u] = w[i < k ? i : k - 1];
      }
#pragma unroll
      for (int u = 0; u < kWp; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int64_t i = wd0 * 64 + 4 * (int64_t)(tid + u * kThreads) + j;
          w4[u][j] = w[i < k ? i : k - 1];
        }
#pragma unroll
      for (int u = 0; u < kZ; ++u) {
        const int idx = tid + u * kThreads, r = idx / kChunk, c = idx - r * kChunk;
        const bool in = wd0 + c < wend;
        As[r][c] = (a0 + r < n && in) ? (za[u] & kp) : 0ull;  // kept rows only
        Bs[r][c] = (b0 + r < n && in) ? zb[u] : 0ull;
      }
#pragma unroll
      for (int u = 0; u < kWr; ++u) {
        const int idx = tid + u * kThreads;
        wrow[idx] = wd0 * 64 + idx < k ? wr_[u] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < kWp; ++u) {  // rows 4 idx .. 4 idx + 3 of the chunk
        const int idx = tid + u * kThreads;
        uint32_t pc[3][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int64_t i = wd0 * 64 + 4 * (int64_t)idx + j;
          float rest = i < k ? w4[u][j] : 0.f;
#pragma unroll
          for (int p = 0; p < 3; ++p) {
            pc[p][j] = bf16_bits_rn(rest);
            rest -= __uint_as_float(pc[p][j] << 16);  // exact: the piece shares the leading bits of `rest`
          }
        }
#pragma unroll
        for (int p = 0; p < 3; ++p) wpk[p][idx] = gram_u2_t{pc[p][0] | (pc[p][1] << 16), pc[p][2] | (pc[p][3] << 16)};
      }
    }
    if (tid < kChunk) {
      const int64_t wd = wd0 + tid;
      wus[tid] = wd < wend ? wu[wd] : 0.f;
      unis[tid] = wd < wend ? uni[wd] : 1;
    }
    __syncthreads();
    float f[4][4];
    for (int i = 0; i < 4; ++i)
      for (int j = 0; j < 4; ++j) f[i][j] = 0.f;
    gram_f16_t fm0, fm1;
#pragma unroll
    for (int i = 0; i < 16; ++i) { fm0[i] = 0.f; fm1[i] = 0.f; }
    for (int c = 0; c < kChunk; ++c) {
      if (unis[c] == 1) {
        uint64_t av[4], bv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          av[i] = As[ty + 16 * i][c];
          bv[i] = Bs[tx + 16 * i][c];
        }
        const float wv = wus[c];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) f[i][j] += wv * (float)__popcll(av[i] & bv[j]);
      } else if (unis[c] == 3) {
        // no kept row in this word
      } else if (unis[c] == 2) {
        // rows 8 kb + 4 half + j, j < 4: a nibble of each column word per step (pre-shifted by 4 half)
        const uint64_t aw = As[wi + l32][c] >> (4 * half), bw = Bs[wj + l32][c] >> (4 * half);
        const gram_u2_t* w1 = wpk[0] + c * 16 + half;
        const gram_u2_t* w2 = wpk[1] + c * 16 + half;
        const gram_u2_t* w3 = wpk[2] + c * 16 + half;
#pragma unroll
        for (int kb = 0; kb < 8; ++kb) {
          const gram_u2_t am = tabA[(uint32_t)(aw >> (8 * kb)) & 15u];
          const gram_s4_t bo = __builtin_bit_cast(gram_s4_t, tabB[(uint32_t)(bw >> (8 * kb)) & 15u]);
          const gram_u2_t p1 = w1[2 * kb], p2 = w2[2 * kb], p3 = w3[2 * kb];
          const gram_s4_t a1 = __builtin_bit_cast(gram_s4_t, gram_u2_t{p1.x & am.x, p1.y & am.y});
          const gram_s4_t a2 = __builtin_bit_cast(gram_s4_t, gram_u2_t{p2.x & am.x, p2.y & am.y});
          const gram_s4_t a3 = __builtin_bit_cast(gram_s4_t, gram_u2_t{p3.x & am.x, p3.y & am.y});
          fm0 = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a1, bo, fm0, 0, 0, 0);
          fm1 = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a2, bo, fm1, 0, 0, 0);
          fm1 = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a3, bo, fm1, 0, 0, 0);
        }
      } else {
        uint64_t av[4], bv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          av[i] = As[ty + 16 * i][c];
          bv[i] = Bs[tx + 16 * i][c];
        }
        const float* wr = wrow + c * 64;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            uint64_t m = av[i] & bv[j];
            float sum = 0.f;
            while (m) {
              sum += wr[__ffsll((long long)m) - 1];
              m &= m - 1;
            }
            f[i][j] += sum;
          }
      }
    }
    for (int i = 0; i < 4; ++i)
      for (int j = 0; j < 4; ++j) acc[i][j] += (double)f[i][j];
#pragma unroll
    for (int i = 0; i < 16; ++i) accm[i] += (double)fm0[i] + (double)fm1[i];
  }
  // merge: the matrix-core quadrants pass through LDS into the popcount path's element order
  __syncthreads();
  double (*Ts)[kTile + 1] = (double (*)[kTile + 1])raw;
#pragma unroll
  for (int i = 0; i < 16; ++i) Ts[wi + 8 * (i / 4) + 4 * half + (i % 4)][wj + l32] = accm[i];
  __syncthreads();
  // slice 0 already holds the sparse rows' part (both triangles): all of a thread's entries are fetched before the
  // first store (one memory latency instead of sixteen; addresses clamped instead of skipped)
  double prev[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t a = a0 + ty + 16 * i, b = b0 + tx + 16 * j;
      prev[i][j] = blockIdx.z == 0 ? G[(a < n ? a : n - 1) * n + (b < n ? b : n - 1)] : 0.0;
    }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t a = a0 + ty + 16 * i, b = b0 + tx + 16 * j;
      if (a < n && b < n) {
        const double v = acc[i][j] + Ts[ty + 16 * i][tx + 16 * j] + prev[i][j];
        G[a * n + b] = v;
        if (ta != tb) G[b * n + a] = v;  // a diagonal tile computes both of its triangles itself
      }
    }
}

// G = sum of the slices (into slice 0) and the row means of G; one workgroup per row (grid-stride)
__global__ __launch_bounds__(kThreads) void sum_slices_row_mean_kernel(double* Gp, int64_t n, int slices, double* m) {
  __shared__ double red[kThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int64_t a = blockIdx.x; a < n; a += gridDim.x) {
    double s = 0.0;
    for (int64_t b = threadIdx.x; b < n; b += kThreads) {
      double g = Gp[a * n + b];
      for (int z = 1; z < slices; ++z) g += Gp[(size_t)z * n * n + a * n + b];
      Gp[a * n + b] = g;
      s += g;
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
      double t = 0.0;
      for (int w = 0; w < kThreads / 64; ++w) t += red[w];  // fixed order
      m[a] = t / (double)n;
    }
    __syncthreads();
  }
}

// single block: stats[0] = mu (grand mean of G), stats[1] = trace(G)
__global__ __launch_bounds__(kThreads) void stats_kernel(const double* G, const double* m, int64_t n, double* stats) {
  __shared__ double sh[2][kThreads];
  double a = 0, b = 0;
  for (int64_t i = threadIdx.x; i < n; i += kThreads) {
    a += m[i];
    b += G[i * n + i];
  }
  sh[0][threadIdx.x] = a;
  sh[1][threadIdx.x] = b;
  __syncthreads();
  if (threadIdx.x == 0) {
    double x = 0, yv = 0;
    for (int i = 0; i < kThreads; ++i) {
      x += sh[0][i];
      yv += sh[1][i];
    }
    stats[0] = x / (double)n;
    stats[1] = yv;
  }
}

// The system lives in one (n+1) x ld array M: rows 0..n-1 = A = P G P + gamma 11^T / n (lower triangle
// is what the factorisation reads), row n = the right-hand side c - mean(c). Factorising with row n
// carried along as an ordinary sub-diagonal row leaves L^-1 rhs in it (the forward solve comes for free).
// gamma = trace(PGP)/(n-1) keeps the added direction at the scale of the other eigenvalues.
// pivot_floor: the smallest pivot the factorisation accepts, relative to the mean diagonal entry of A: a pivot
// that exact arithmetic would make zero (a direction the sampled rows do not determine) comes out of fp64
// as about n * 2^-52 times the scale, with either sign; 256 n 2^-52 sits well above that and far below the
// pivots of a determined system.
__global__ void build_matrix_kernel(const double* G, const double* m, const double* stats, int64_t n, int64_t ld, double* M,
                                    double* pivot_floor) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n * n) return;
  const double mu = stats[0];
  const double tr = stats[1] - (double)n * mu;
  double gamma = tr / (double)(n > 1 ? n - 1 : 1);
  if (!(gamma > 0.0)) gamma = 1.0;
  if (idx == 0) *pivot_floor = 256.0 * (double)n * 0x1p-52 * ((tr > 0.0 ? tr : 0.0) + gamma) / (double)n;
  const int64_t a = idx / n, b = idx - a * n;
  M[a * ld + b] = G[idx] - m[a] - m[b] + mu + gamma / (double)n;
}

// row n of M = c - mean(c); single block
__global__ __launch_bounds__(kThreads) void build_rhs_kernel(const double* c, int64_t n, int64_t ld, double* M) {
  __shared__ double sh[kThreads];
  double a = 0;
  for (int64_t i = threadIdx.x; i < n; i += kThreads) a += c[i];
  sh[threadIdx.x] = a;
  __syncthreads();
  if (threadIdx.x == 0) {
    double x = 0;
    for (int i = 0; i < kThreads; ++i) x += sh[i];
    sh[0] = x / (double)n;
  }
  __syncthreads();
  const double mean = sh[0];
  for (int64_t i = threadIdx.x; i < n; i += kThreads) M[n * ld + i] = c[i] - mean;
}

// ---------------- blocked Cholesky (lower, in place, fp64) ----------------
constexpr int NB = 64;
constexpr int64_t kSuperCols = 256;  // columns of a super-panel (large trailing matrices)

// 1/sqrt(p) for 1e-30 < p < 1e30: single-precision seed, two Newton steps r += r (1/2 - (p/2) r^2) in double (a
// short dependent chain; the library routine costs several times more per step of a sequential loop)
__device__ __forceinline__ double fast_rsqrt(double p) {
  double r = (double)__frsqrt_rn((float)p);  // relative error about 1e-7
  const double hp = 0.5 * p;
  r = fma(r, fma(-hp * r, r, 0.5), r);        // -> 1e-14
  r = fma(r, fma(-hp * r, r, 0.5), r);        // -> below one ulp
  return r;
}

// 1/p for 1e-30 < p < 1e30: hardware seed (about 24 bits), two Newton steps x += x (1 - p x)
__device__ __forceinline__ double fast_rcp(double p) {
  double x = __builtin_amdgcn_rcp(p);
  x = fma(x, fma(-p, x, 1.0), x);
  x = fma(x, fma(-p, x, 1.0), x);
  return x;
}

typedef double double4_t __attribute__((ext_vector_type(4)));

// acc (+)= A[64 x 64] * B[64 x 64]^T for 64x64 tiles held in LDS with row pitch NB+1, on the fp64
// matrix cores. Each of the four waves owns a 32x32 quadrant = 2x2 tiles of v_mfma_f64_16x16x4f64:
// lane l supplies A[i = l%16][k = l/16] and B^T[k = l/16][j = l%16] = B[j][k]; its four results are
// D[4*r + l/16][l%16], r = 0..3.
__device__ __forceinline__ void tile_nt_mfma(const double (*A)[NB + 1], const double (*B)[NB + 1], double4_t (&acc)[2][2]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;
  const int l16 = lane & 15, lk = lane >> 4;
  const double* pa0 = &A[wi + l16][lk];
  const double* pa1 = &A[wi + 16 + l16][lk];
  const double* pb0 = &B[wj + l16][lk];
  const double* pb1 = &B[wj + 16 + l16][lk];
  // the operands of the next step are read from LDS before this step's products are issued
  double a0 = pa0[0], a1 = pa1[0], b0 = pb0[0], b1 = pb1[0];
#pragma unroll
  for (int k0 = 0; k0 < NB; k0 += 4) {
    double na0 = 0.0, na1 = 0.0, nb0 = 0.0, nb1 = 0.0;
    if (k0 + 4 < NB) {
      na0 = pa0[k0 + 4];
      na1 = pa1[k0 + 4];
      nb0 = pb0[k0 + 4];
      nb1 = pb1[k0 + 4];
    }
    acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
    a0 = na0;
    a1 = na1;
    b0 = nb0;
    b1 = nb1;
  }
}

// A 64 x 64 tile from global memory into LDS (row pitch NB+1) in two halves, so that a kernel can have the loads of
// all its tiles in flight before the first LDS store: written as one loop that loads and stores element by element
// (the bounds checks make every load a branch of its own), each of a thread's 16 elements costs a memory latency.
// Element (r, c) is src[(row0 + r) * stride + col0 + c], valid for row0 + r < row_limit and c < ncols, zero otherwise;
// out-of-range elements are read from a clamped address. row_limit and ncols are at least 1.
struct TileRegs {
  double v[kTile * NB / kThreads];
};
__device__ __forceinline__ void tile_fetch(TileRegs& t, const double* src, int64_t stride, int64_t row0, int64_t row_limit,
                                           int64_t col0, int ncols) {
#pragma unroll
  for (int u = 0; u < kTile * NB / kThreads; ++u) {
    const int idx = threadIdx.x + u * kThreads, r = idx >> 6, c = idx & 63;
    const int64_t rr = row0 + r < row_limit ? row0 + r : row_limit - 1;
    t.v[u] = src[rr * stride + col0 + (c < ncols ? c : ncols - 1)];
  }
}
__device__ __forceinline__ void tile_put(double (*T)[NB + 1], const TileRegs& t, int64_t row0, int64_t row_limit, int ncols) {
#pragma unroll
  for (int u = 0; u < kTile * NB / kThreads; ++u) {
    const int idx = threadIdx.x + u * kThreads, r = idx >> 6, c = idx & 63;
    T[r][c] = (row0 + r < row_limit && c < ncols) ? t.v[u] : 0.0;
  }
}

// M[r][c] -= acc over a wave's NI x NJ matrix-core tiles at (i0 + wi, c0 + wj), lower triangle and in-bounds
// entries only; P, if not null, also receives the new values of the tile's column block (row r at P[r * 64 ..]).
// All loads of a tile row are issued before the first store: written as `M[..] -= acc` under its bounds check,
// every entry becomes a load, a wait and a store of its own, one memory latency each. The loads are made safe
// by clamping the address instead of skipping them.
template <int NI, int NJ>
__device__ __forceinline__ void tile_sub_store(double* M, int64_t ld, int64_t rows_total, int64_t n, int64_t i0, int64_t c0,
                                               int wi, int wj, const double4_t (&acc)[NI][NJ], double* P) {
  const int lane = threadIdx.x & 63, l16 = lane & 15, lk = lane >> 4;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    double cur[NJ][4];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int64_t r = i0 + wi + 16 * i + 4 * r4 + lk, c = c0 + wj + 16 * j + l16;
        const int64_t rs = r < rows_total ? r : rows_total - 1, cs = c < n ? c : n - 1;
        cur[j][r4] = M[rs * ld + cs];
      }
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int64_t r = i0 + wi + 16 * i + 4 * r4 + lk, c = c0 + wj + 16 * j + l16;
        if (r < rows_total && c < n && c <= r) {
          const double v = cur[j][r4] - acc[i][j][r4];
          M[r * ld + c] = v;
          if (P) P[r * NB + (c - c0)] = v;
        }
      }
  }
}

// value of `v` in lane `src` (a compile-time constant after unrolling) for the whole wave, through two scalar registers
__device__ __forceinline__ double wave_bcast(double v, int src) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
  return __hiloint2double(hi, lo);
}

constexpr int kSub = 16;  // sub-block of the diagonal block: one matrix-core tile

// One wave eliminates the 16 x 16 block D = S[o.., o..] and, alongside, the identity: what it leaves is the factor
// and its inverse up to the scaling by 1/sqrt(pivot), which the other waves apply where they use them,
//   L[i][k] = S[o+i][o+k] r_k,   Linv[k][c] = XT[c][k] r_k,   r_k = 1/sqrt(d_k),   d_k = S[o+k][o+k].
// A lone wave issues one instruction every few cycles whatever the instruction is, so the loop holds nothing that
// can be done elsewhere: no square root, no pivot check, no stores to global memory.
// Lane l < 16 keeps row l of D (columns up to l matter), lane 16 + l keeps column l of the inverse (the upper half
// of the wave repeats the lower). With d the pivot of column j and p = 1/d, L[i][j] L[k][j] = S[i][j] S[k][j] p:
// lane i subtracts (S[i][j] p) col[k] from its entry of column k > j, where col[] is column j as updated so far,
// which every lane has put into LDS (entry j of it is the pivot's own lane's); the same column moves the forward substitution L X = I on,
// X[k][c] -= col[k] (X[j][c] p), so one multiply-add per k serves both halves. The pivot reaches all lanes through
// scalar registers; the column travels through LDS (two buffers; reads of one address by all lanes are a
// broadcast) under the updates of the step before. I16 is a 16 x 16 identity.
__device__ __forceinline__ void eliminate_sub_block(double (*S)[NB + 1], int o, double (*XT)[kSub + 1],
                                                    const double (*I16)[kSub + 1], double* col) {
  const int lane = threadIdx.x & 63, l = lane & 15, slot = lane & 31;
  const bool inv = (lane & 16) != 0;
  double* mine = inv ? &XT[l][0] : &S[o + l][o];
  const double* init = inv ? &I16[l][0] : mine;
  double v[kSub];
#pragma unroll
  for (int k = 0; k < kSub; ++k) v[k] = init[k];
  // The column's store and loads are written as instructions: the loads of the next column have to be issued right
  // behind its store, so that they return under the remaining updates of this column, and the compiler's scheduler
  // puts them next to their first use instead. LDS answers a wave in order, so the compiler's own counting of its
  // LDS accesses stays on the safe side. Between a load and the wait below its destination registers are in flight,
  // which the compiler does not know: tests/test_isa_lds_reads.py checks the generated code for any use in between.
  typedef double pair_t __attribute__((ext_vector_type(2)));
  const unsigned col_lds = (unsigned)(size_t)(__attribute__((address_space(3))) double*)col;  // byte address in LDS
  const unsigned slot_lds = col_lds + 8u * slot;
  pair_t q[kSub / 2];
  asm volatile("ds_write_b64 %0, %1" ::"v"(slot_lds), "v"(v[0]) : "memory");
#pragma unroll
  for (int h = 0; h < kSub / 2; ++h) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(q[h]) : "v"(col_lds), "n"(16 * h));
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3]), "+v"(q[4]), "+v"(q[5]), "+v"(q[6]), "+v"(q[7]));
  double c[kSub];
#pragma unroll
  for (int h = 0; h < kSub / 2; ++h) {
    c[2 * h] = q[h].x;
    c[2 * h + 1] = q[h].y;
  }
#pragma unroll
  for (int j = 0; j + 1 < kSub; ++j) {
    const double p = v[j] * fast_rcp(wave_bcast(v[j], j));
    v[j + 1] = fma(-p, c[j + 1], v[j + 1]);
    if (j + 2 < kSub) {  // the next column is complete: send it on its way before the other updates
      asm volatile("ds_write_b64 %0, %1 offset:%2" ::"v"(slot_lds), "v"(v[j + 1]), "n"(((j + 1) & 1) * 256) : "memory");
#pragma unroll
      for (int h = (j + 2) / 2; h < kSub / 2; ++h)
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(q[h]) : "v"(col_lds), "n"(((j + 1) & 1) * 256 + 16 * h));
    }
#pragma unroll
    for (int k = j + 2; k < kSub; ++k) v[k] = fma(-p, c[k], v[k]);
    // pin the updates to this step: left to itself the compiler defers the updates of a column until the column's
    // own step and holds every earlier column in registers for them
#pragma unroll
    for (int k = j + 2; k < kSub; ++k) asm volatile("" : "+v"(v[k]));
    if (j + 2 < kSub) {
      // q[h] for h below (j + 2) / 2 were not loaded again and pass through unchanged
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3]), "+v"(q[4]), "+v"(q[5]), "+v"(q[6]), "+v"(q[7]));
#pragma unroll
      for (int h = (j + 2) / 2; h < kSub / 2; ++h) {
        c[2 * h] = q[h].x;
        c[2 * h + 1] = q[h].y;
      }
    }
  }
  asm volatile("" ::: "memory");
#pragma unroll
  for (int k = 0; k < kSub; ++k) mine[k] = v[k];
}

// sum_k A(m, k) B(k, n) over a 16 x 16 x 16 product on the fp64 matrix cores, added to acc: A(m, k) = Ap[m * ars + k * acs]
// and B(k, n) = Bp[k * brs + n * bcs]; lane l holds D[4 r + l / 16][l % 16], r = 0..3.
__device__ __forceinline__ double4_t sub_block_mma(const double* Ap, int ars, int acs, const double* Bp, int brs, int bcs,
                                                   double4_t acc) {
  const int lane = threadIdx.x & 63, l16 = lane & 15, lk = lane >> 4;
#pragma unroll
  for (int kk = 0; kk < kSub; kk += 4) {
    const double av = Ap[l16 * ars + (kk + lk) * acs];
    const double bv = Bp[(kk + lk) * brs + l16 * bcs];
    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
  }
  return acc;
}
__device__ __forceinline__ double4_t sub_block_load(const double (*T)[NB + 1], int r0, int c0) {
  const int lane = threadIdx.x & 63, l16 = lane & 15, lk = lane >> 4;
  double4_t v;
#pragma unroll
  for (int r = 0; r < 4; ++r) v[r] = T[r0 + 4 * r + lk][c0 + l16];
  return v;
}
__device__ __forceinline__ void sub_block_store(double (*T)[NB + 1], int r0, int c0, double4_t v) {
  const int lane = threadIdx.x & 63, l16 = lane & 15, lk = lane >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r) T[r0 + 4 * r + lk][c0 + l16] = v[r];
}

// Factor the nb x nb diagonal block at j0 (lower factor L, in place) and invert the factor: Linv (NB x NB,
// identity-padded) goes to linv_out. One workgroup of four waves; the block S and the inverse Y live in the two
// LDS tiles the caller hands over. The block is taken as 4 x 4 sub-blocks of 16, left-looking; for block column b
//   A. S_ib -= sum_{k<b} L_ik L_bk^T for i >= b, and T_bj = sum_{j<=k<b} L_bk Y_kj for j < b   (4 tasks, one a wave),
//   B. one wave eliminates S_bb and the identity beside it (the only sequential part: 16 columns),
//   C. L_ib = S_ib Linv_bb^T for i > b, Y_bj = -Linv_bb T_bj for j < b, and the scaled L_bb and Y_bb = Linv_bb
//      (4 tasks, one a wave; this is where the square roots are taken and the pivots are checked),
// where Y follows the forward substitution L Y = I block row by block row. A and C are 16 x 16 x 16 products on the
// fp64 matrix cores; results go to global memory as they appear. A pivot that is not positive (or not a number, or
// below the relative floor stored next to the flag, or above 1e30) raises the flag; nothing is repaired, the caller discards a flagged factorisation.
// `pend`: optional 64 x 64 tile (LDS, pitch NB+1; may be the tile Y) holding the rows of this block in the panel
// just finished; its outer product is the one trailing update the block has not received yet and is subtracted
// first.
// the block's entries as chol_diag_body wants them (identity beyond nb): each wave's 32 x 32 quadrant, matrix-core
// layout. A caller with other work to do first loads them early, so that they arrive under that work.
__device__ __forceinline__ void load_diag_block(const double* M, int64_t ld, int64_t j0, int nb, double4_t (&mt)[2][2]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int r = wi + 16 * i + 4 * r4 + (lane >> 4), c = wj + 16 * j + (lane & 15);
        mt[i][j][r4] = (r < nb && c < nb) ? M[(j0 + r) * ld + j0 + c] : (r == c ? 1.0 : 0.0);
      }
}

__device__ __forceinline__ void chol_diag_body(double* M, int64_t ld, int64_t j0, int nb, double* linv_out, int* flag,
                                               const double (*pend)[NB + 1], double (*S)[NB + 1], double (*Y)[NB + 1],
                                               const double4_t (&mt)[2][2]) {
  __shared__ double XT[kSub][kSub + 1];
  __shared__ double I16[kSub][kSub + 1];
  __shared__ __align__(16) double col[2 * 32];  // two buffers for the column in flight
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lk = lane >> 4;
  {
    double4_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = double4_t{0.0, 0.0, 0.0, 0.0};
    if (pend) {  // rows past nb of the tile are zero, so the identity padding stays as it is
      tile_nt_mfma(pend, pend, acc);
      __syncthreads();  // every wave has read `pend` before Y (possibly the same tile) is written
    }
    const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int r = wi + 16 * i + 4 * r4 + lk, c = wj + 16 * j + l16;
          S[r][c] = mt[i][j][r4] - acc[i][j][r4];
        }
    I16[tid >> 4][tid & 15] = (tid >> 4) == (tid & 15) ? 1.0 : 0.0;
    // the sub-blocks of Linv above the diagonal are zero; the others are written as they are computed
    for (int idx = tid; idx < NB * NB; idx += kThreads)
      if (((idx & 63) >> 4) > (idx >> 10)) linv_out[idx] = 0.0;
  }
  __syncthreads();
  constexpr int nsb = NB / kSub;
  const double4_t zero = double4_t{0.0, 0.0, 0.0, 0.0};
  for (int b = 0; b < nsb; ++b) {
    const int o = b * kSub;
    if (b > 0) {  // A
      if (wave < nsb - b) {
        const int i = b + wave;
        double4_t acc = zero;
        for (int k = 0; k < b; ++k)  // (m, n): sum_kk S[16 i + m][16 k + kk] S[16 b + n][16 k + kk]
          acc = sub_block_mma(&S[i * kSub][k * kSub], NB + 1, 1, &S[o][k * kSub], 1, NB + 1, acc);
        sub_block_store(S, i * kSub, o, sub_block_load(S, i * kSub, o) - acc);
      } else {
        const int j = wave - (nsb - b);
        double4_t acc = zero;
        for (int k = j; k < b; ++k)  // (m, n): sum_kk S[o + m][16 k + kk] Y[16 k + kk][16 j + n]
          acc = sub_block_mma(&S[o][k * kSub], NB + 1, 1, &Y[k * kSub][j * kSub], NB + 1, 1, acc);
        sub_block_store(Y, o, j * kSub, acc);
      }
      __syncthreads();
    }
    if (wave == 0) eliminate_sub_block(S, o, XT, I16, col);  // B
    __syncthreads();
    {  // C
      const double d = S[o + l16][o + l16];
      const double rl = fast_rsqrt(d);  // r of this lane's column; r of row m is lane m's
      if (wave < nsb - 1 - b) {
        const int i = b + 1 + wave;  // L_ib(m, n) = r_n sum_k S_ib(m, k) XT(k, n)
        const double4_t xv = sub_block_mma(&S[i * kSub][o], NB + 1, 1, &XT[0][0], kSub + 1, 1, zero) * rl;
        sub_block_store(S, i * kSub, o, xv);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = i * kSub + 4 * r + lk;
          if (row < nb) M[(j0 + row) * ld + j0 + o + l16] = xv[r];
        }
      } else if (wave < nsb - 1) {
        const int j = wave - (nsb - 1 - b);  // Y_bj(m, n) = -r_m sum_k XT(k, m) T(k, n)
        const double4_t tv = sub_block_mma(&XT[0][0], 1, kSub + 1, &Y[o][j * kSub], NB + 1, 1, zero);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const double yv = -tv[r] * __shfl(rl, 4 * r + lk);
          Y[o + 4 * r + lk][j * kSub + l16] = yv;
          linv_out[(o + 4 * r + lk) * NB + j * kSub + l16] = yv;
        }
      } else {
        if (!(d > *(const double*)(flag + 2) && d < 1e30)) atomicExch(flag, 1);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int m = 4 * r + lk;  // row of the sub-block, column l16
          const double x = XT[l16][m] * __shfl(rl, m);
          Y[o + m][o + l16] = x;
          linv_out[(o + m) * NB + o + l16] = x;
          if (l16 <= m && o + m < nb) M[(j0 + o + m) * ld + j0 + o + l16] = S[o + m][o + l16] * rl;
        }
      }
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(kThreads) void chol_diag_kernel(double* M, int64_t ld, int64_t j0, int nb, double* linv_out,
                                                             int* flag) {
  __shared__ double S[kTile][NB + 1];
  __shared__ double Y[kTile][NB + 1];
  double4_t mt[2][2];
  load_diag_block(M, ld, j0, nb, mt);
  chol_diag_body(M, ld, j0, nb, linv_out, flag, nullptr, S, Y, mt);
}

// rows below the diagonal block: X = A21 L11^-T = A21 Linv^T, a 64x64 product per workgroup
__global__ __launch_bounds__(kThreads) void chol_panel_kernel(double* M, int64_t ld, int64_t rows_total, int64_t j0,
                                                              int nb, const double* linv) {
  __shared__ double As[kTile][NB + 1];
  __shared__ double Ls[NB][NB + 1];
  const int64_t i0 = j0 + nb + (int64_t)blockIdx.x * kTile;
  {
    TileRegs ta, tl;
    tile_fetch(ta, M, ld, i0, rows_total, j0, nb);
    tile_fetch(tl, linv, NB, 0, NB, 0, NB);
    tile_put(As, ta, i0, rows_total, nb);
    tile_put(Ls, tl, 0, NB, NB);
  }
  __syncthreads();
  double4_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = double4_t{0.0, 0.0, 0.0, 0.0};
  tile_nt_mfma(As, Ls, acc);
  {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int64_t r = i0 + wi + 16 * i + 4 * r4 + (lane >> 4);
          const int c = wj + 16 * j + (lane & 15);
          if (r < rows_total && c < nb) M[r * ld + j0 + c] = acc[i][j][r4];
        }
  }
}

// trailing update A22 -= L21 L21^T on the lower tiles (rows up to rows_total, columns below n).
// The workgroup of the first diagonal tile does more: that tile is the next diagonal block, so it applies the
// tile's update in registers and factorises it straight away (and stores its inverse), while the other
// workgroups are still updating the rest of the trailing matrix. The next step then starts at its panel.
// (FUSE = false: plain update of every tile; used while the trailing matrix is large, where the registers of
// the factorisation would halve the number of resident update workgroups for no gain.)
template <bool FUSE>
__global__ __launch_bounds__(kThreads) void chol_update_kernel(double* M, int64_t ld, int64_t rows_total, int64_t n,
                                                               int64_t j0, int nb, double* linv_next, int* flag) {
  const int ti = blockIdx.y, tj = blockIdx.x;
  if (tj > ti) return;
  __shared__ double Li[kTile][NB + 1];
  __shared__ double Lj[kTile][NB + 1];
  const int64_t base = j0 + nb;
  const int64_t i0 = base + (int64_t)ti * kTile, c0 = base + (int64_t)tj * kTile;
  {
    TileRegs ta, tb;
    tile_fetch(ta, M, ld, i0, rows_total, j0, nb);
    tile_fetch(tb, M, ld, c0, n, j0, nb);
    tile_put(Li, ta, i0, rows_total, nb);
    tile_put(Lj, tb, c0, n, nb);
  }
  __syncthreads();
  if (FUSE && ti == 0 && tj == 0) {  // Lj holds the rows of the next diagonal block in this panel (zero past column n)
    // a short last block shares its tile with the right-hand-side row, which still needs this update
    if (n - base < NB && (int64_t)threadIdx.x < n - base) {
      const int rr = (int)(n - base), c = threadIdx.x;
      double sum = 0.0;
      for (int k = 0; k < NB; ++k) sum += Li[rr][k] * Lj[c][k];
      M[n * ld + base + c] -= sum;
    }
    __syncthreads();  // the row above has read Li, which becomes the block's tile
    double4_t mt[2][2];
    load_diag_block(M, ld, base, (int)(n - base < NB ? n - base : NB), mt);
    chol_diag_body(M, ld, base, (int)(n - base < NB ? n - base : NB), linv_next, flag, Lj, Li, Lj, mt);
    return;
  }
  double4_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = double4_t{0.0, 0.0, 0.0, 0.0};
  tile_nt_mfma(Li, Lj, acc);
  {
    const int wave = threadIdx.x >> 6;
    tile_sub_store<2, 2>(M, ld, rows_total, n, i0, c0, (wave >> 1) * 32, (wave & 1) * 32, acc, nullptr);
  }
}

// One launch per 64-column step while the trailing matrix is small (at most kFuseMaxRows rows): panel solve,
// trailing update and factorisation of the next diagonal block together. Every workgroup (ti, tj), tj <= ti, first
// solves its own two 64-row pieces of the panel, X = A Linv^T, instead of waiting for a launch that does so
// (twice the arithmetic of the update itself, on workgroups that would otherwise be idle), then updates its tile;
// the workgroup of the first diagonal tile factorises that tile instead, as in chol_update_kernel<true>.
// The rows of the panel as the step before left them come from Pcur (row r of the matrix at Pcur[r * 64 ..]), not
// from M: the workgroups of tile column 0 store the solved panel to M while others may still be reading, and they
// store their updated tile, the next step's panel, to Pnext as well.
__global__ __launch_bounds__(kThreads) void chol_step_kernel(double* M, int64_t ld, int64_t rows_total, int64_t n, int64_t j0,
                                                             const double* linv, double* linv_next, int* flag,
                                                             const double* Pcur, double* Pnext) {
  const int ti = blockIdx.y, tj = blockIdx.x;
  if (tj > ti) return;
  __shared__ double Li[kTile][NB + 1];
  __shared__ double Lj[kTile][NB + 1];
  __shared__ double Ls[NB][NB + 1];
  const int64_t base = j0 + NB;
  const int64_t i0 = base + (int64_t)ti * kTile, c0 = base + (int64_t)tj * kTile;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wi = (wave >> 1) * 32, wj = (wave & 1) * 32;
  double4_t mt[2][2];  // the next diagonal block (first diagonal tile only), on its way while the panel is solved
  if (ti == 0) load_diag_block(M, ld, base, (int)(n - base < NB ? n - base : NB), mt);
  {
    TileRegs ta, tb, tl;
    tile_fetch(ta, Pcur, NB, i0, rows_total, 0, NB);
    tile_fetch(tl, linv, NB, 0, NB, 0, NB);
    if (ti != tj) tile_fetch(tb, Pcur, NB, c0, rows_total, 0, NB);  // tj < ti: all 64 rows lie above row i0 <= n
    tile_put(Li, ta, i0, rows_total, NB);
    tile_put(Ls, tl, 0, NB, NB);
    if (ti != tj) tile_put(Lj, tb, c0, rows_total, NB);
  }
  __syncthreads();
  double4_t xi[2][2], xj[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) xi[i][j] = xj[i][j] = double4_t{0.0, 0.0, 0.0, 0.0};
  tile_nt_mfma(Li, Ls, xi);
  if (ti != tj) tile_nt_mfma(Lj, Ls, xj);
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int r = wi + 16 * i + 4 * r4 + (lane >> 4), c = wj + 16 * j + (lane & 15);
        const double x = xi[i][j][r4];
        Li[r][c] = x;
        // on a diagonal tile Lj is the same piece without the right-hand-side row (row n of the matrix)
        Lj[r][c] = ti != tj ? xj[i][j][r4] : (c0 + r < n ? x : 0.0);
        if (tj == 0 && i0 + r < rows_total) M[(i0 + r) * ld + j0 + c] = x;
      }
  __syncthreads();
  if (ti == 0) {  // tj == 0 too: the next diagonal block
    // a short last block shares its tile with the right-hand-side row, which still needs this update
    if (n - base < NB && (int64_t)threadIdx.x < n - base) {
      const int rr = (int)(n - base), c = threadIdx.x;
      double sum = 0.0;
      for (int k = 0; k < NB; ++k) sum += Li[rr][k] * Lj[c][k];
      M[n * ld + base + c] -= sum;
    }
    __syncthreads();  // the row above has read Li, which becomes the block's tile
    chol_diag_body(M, ld, base, (int)(n - base < NB ? n - base : NB), linv_next, flag, Lj, Li, Ls, mt);
    return;
  }
  double4_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = double4_t{0.0, 0.0, 0.0, 0.0};
  tile_nt_mfma(Li, Lj, acc);
  tile_sub_store<2, 2>(M, ld, rows_total, n, i0, c0, wi, wj, acc, tj == 0 ? Pnext : nullptr);
}

// rows [row0, rows_total) of the 64 columns at j0 -> P (row r at P[r * 64 ..]): the panel of the first fused step
__global__ void copy_panel_kernel(const double* M, int64_t ld, int64_t rows_total, int64_t row0, int64_t j0, int64_t n, double* P) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t r = row0 + (idx >> 6);
  const int c = (int)(idx & 63);
  if (r < rows_total) P[r * NB + c] = j0 + c < n ? M[r * ld + j0 + c] : 0.0;
}

// Trailing update of a whole super-panel: A22 -= L21 L21^T with L21 = the kw (a multiple of 64) columns
// starting at J, on the lower 64x64 tiles of the matrix from row/column `base` = J + kw on. The tile stays in
// registers across the kw/64 column chunks, so it is read and written once per super-panel instead of once
// per 64 columns; the next chunk of the two operands is fetched into registers while the matrix cores work on
// the current one.
template <int KW>  // columns of the super-panel: known at compile time, so that the chunk loop unrolls (column offsets
                   // become immediates and the accumulators stay where the matrix cores want them)
__global__ __launch_bounds__(kThreads) void chol_update_wide_kernel(double* M, int64_t ld, int64_t rows_total, int64_t n,
                                                                    int64_t J, int64_t base) {
  constexpr int kw = KW;
  const int ti = blockIdx.y, tj = blockIdx.x;
  if (tj > ti) return;
  __shared__ double Li[kTile][NB + 1];
  __shared__ double Lj[kTile][NB + 1];
  const int tid = threadIdx.x;
  const int64_t i0 = base + (int64_t)ti * kTile, c0 = base + (int64_t)tj * kTile;
  constexpr int kPer = kTile * NB / kThreads;
  double pi[kPer], pj[kPer];
  // Rows past the end of the matrix are read from the last valid row instead of being zeroed: such a row of an
  // operand only reaches rows (or columns) of the tile that are never stored. The row addresses are formed once.
  const double* rowi[kPer];
  const double* rowj[kPer];
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int idx = tid + u * kThreads, r = idx >> 6, c = idx & 63;
    rowi[u] = M + (i0 + r < rows_total ? i0 + r : rows_total - 1) * ld + J + c;
    rowj[u] = M + (c0 + r < n ? c0 + r : n - 1) * ld + J + c;
  }
  auto fetch = [&](int kc) {
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      pi[u] = rowi[u][kc];
      pj[u] = rowj[u][kc];
    }
  };
  double4_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = double4_t{0.0, 0.0, 0.0, 0.0};
  fetch(0);
#pragma unroll
  for (int kc = 0; kc < kw; kc += NB) {
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const int idx = tid + u * kThreads, r = idx >> 6, c = idx & 63;
      Li[r][c] = pi[u];
      Lj[r][c] = pj[u];
    }
    __syncthreads();
    if (kc + NB < kw) fetch(kc + NB);
    tile_nt_mfma(Li, Lj, acc);
  }
  const int wave = tid >> 6;
  tile_sub_store<2, 2>(M, ld, rows_total, n, i0, c0, (wave >> 1) * 32, (wave & 1) * 32, acc, nullptr);
}


// L^T psi = y (y = row n of M after the factorisation), block by block from the end, using the stored
// inverses of the diagonal blocks. One launch per block: every workgroup recomputes the 64 unknowns of
// the block, psi_c = sum_{r >= c} Linv[r][c] y_r (cheap; workgroup 0 stores them), and removes their
// contribution from its own slice of the earlier entries, y_j -= sum_r L[j0+r][j] psi_r.
__global__ __launch_bounds__(kThreads) void chol_back_step_kernel(const double* M, int64_t ld, int64_t j0, int nb,
                                                                  const double* linv, double* yv, double* psi) {
  __shared__ double xs[NB];
  __shared__ double part[kThreads / NB][NB];
  const int tid = threadIdx.x;
  {
    const int c = tid & (NB - 1), q = tid / NB;  // four partial sums per unknown, added in a fixed order
    double s = 0.0;
    for (int r = c + q; r < nb; r += kThreads / NB) s += linv[r * NB + c] * yv[j0 + r];
    part[q][c] = s;
  }
  __syncthreads();
  if (tid < NB) {
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < kThreads / NB; ++q) s += part[q][tid];
    xs[tid] = s;
    if (blockIdx.x == 0 && tid < nb) psi[j0 + tid] = s;
  }
  __syncthreads();
  const int64_t j = (int64_t)blockIdx.x * kThreads + tid;
  if (j < j0) {  // all NB loads of the column are in flight together (rows past a short block are skipped)
    double mv[NB];
#pragma unroll
    for (int r = 0; r < NB; ++r) mv[r] = r < nb ? M[(j0 + r) * ld + j] : 0.0;
    double s = 0.0;
#pragma unroll
    for (int r = 0; r < NB; ++r) s += mv[r] * xs[r];
    yv[j] -= s;
  }
}

// The same back substitution for small systems (n <= kBackSmallMax) in ONE launch: a single workgroup of
// 512 threads keeps the right-hand side in LDS and walks the blocks from the end; per block the 64 unknowns
// come from the stored inverse (8 partial sums each, added in a fixed order), then every earlier entry
// drops their contribution. At this size the chain of per-block launches costs more than the arithmetic.
constexpr int kBackSmallMax = 2048;
constexpr int64_t kFuseMaxRows = 2048;
constexpr int kBackThreads = 512;
__global__ __launch_bounds__(kBackThreads) void chol_back_small_kernel(const double* M, int64_t ld, int64_t n, int nblk,
                                                                       const double* linv, const float* y01, float* phi) {
  __shared__ double ys[kBackSmallMax];
  __shared__ double xs[NB];
  __shared__ double part[kBackThreads / NB][NB];
  const int tid = threadIdx.x;
  for (int j = tid; j < n; j += kBackThreads) ys[j] = M[n * ld + j];
  const double shift = ((double)y01[1] - (double)y01[0]) / (double)n;
  __syncthreads();
  // entries of the block inverse this thread multiplies: column c, rows c + q + 16 i (fetched one block ahead,
  // so that the only memory wait inside a step is the update's own)
  constexpr int kLi = NB / (kBackThreads / NB);
  const int c = tid & (NB - 1), q = tid / NB;
  double lv[kLi];
  auto fetch_li = [&](int bk) {
    const double* li = linv + (size_t)bk * NB * NB;
#pragma unroll
    for (int i = 0; i < kLi; ++i) {
      const int r = c + q + (kBackThreads / NB) * i;
      lv[i] = r < NB ? li[r * NB + c] : 0.0;  // rows past a short last block are skipped in the product
    }
  };
  fetch_li(nblk - 1);
  for (int bk = nblk - 1; bk >= 0; --bk) {
    const int j0 = bk * NB;
    const int nb = (int)(n - j0 < NB ? n - j0 : NB);
    {
      double s = 0.0;
#pragma unroll
      for (int i = 0; i < kLi; ++i) {
        const int r = c + q + (kBackThreads / NB) * i;
        if (r < nb) s += lv[i] * ys[j0 + r];
      }
      part[q][c] = s;
    }
    if (bk > 0) fetch_li(bk - 1);
    __syncthreads();
    if (tid < NB) {
      double s = 0.0;
#pragma unroll
      for (int qq = 0; qq < kBackThreads / NB; ++qq) s += part[qq][tid];
      xs[tid] = s;
      if (tid < nb) phi[j0 + tid] = (float)(s + shift);
    }
    __syncthreads();
    for (int j = tid; j < j0; j += kBackThreads) {
      double s = 0.0;
      const double* mp = M + (size_t)j0 * ld + j;
#pragma unroll 32
      for (int r = 0; r < NB; ++r) s += (r < nb ? mp[(size_t)r * ld] : 0.0) * xs[r];
      ys[j] -= s;
    }
    __syncthreads();
  }
}

__global__ void copy_row_kernel(const double* M, int64_t ld, int64_t n, double* yv) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) yv[j] = M[n * ld + j];
}

__global__ void finish_phi_kernel(const double* psi, const float* y01, int64_t n, float* phi) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const double delta = (double)y01[1] - (double)y01[0];
  phi[j] = (float)(psi[j] + delta / (double)n);
}

inline float dense_fraction(const ds_ctx* ctx) {
  return ctx->tuning.gram_dense_fraction > 0.f ? ctx->tuning.gram_dense_fraction : kDenseFraction;
}
inline int sparse_divisor(const ds_ctx* ctx) {
  return ctx->tuning.gram_sparse_div >= 1 ? ctx->tuning.gram_sparse_div : kSparseDivisor;
}

inline unsigned nblocks(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

struct GramDims {
  int64_t R, RW, ld, nblk;
  int slices;
  int64_t words_per_slice;
};

GramDims gram_dims(int64_t n, int64_t k, int paired, int num_cus) {
  GramDims d;
  d.R = paired ? k / 2 : k;
  d.RW = (d.R + 63) / 64;
  d.ld = (n + 1 + 7) & ~(int64_t)7;
  d.nblk = (n + NB - 1) / NB;
  const int64_t tiles = (n + kTile - 1) / kTile;
  const int64_t lower = tiles * (tiles + 1) / 2;
  if (num_cus > 256) num_cus = 256;
  int64_t s = (2 * (int64_t)num_cus + lower - 1) / lower;
  const int64_t chunks = (d.RW + kChunk - 1) / kChunk;
  if (s > chunks) s = chunks;
  if (s > 16) s = 16;
  if (s < 1) s = 1;
  const int64_t cps = (chunks + s - 1) / s;  // chunks per slice
  d.words_per_slice = cps * kChunk;
  d.slices = (int)((chunks + cps - 1) / cps);
  return d;
}

}  // namespace

// rows of a 64-column panel, one buffer (the fused steps of the factorisation keep two)
static size_t panel_bytes(int64_t n) { return (size_t)(n + 1) * NB * 8; }

size_t ds_gram_arena_bytes(int64_t n, int64_t k) {
  const GramDims d = gram_dims(n, k, 0, 256);  // the unpaired layout is the larger one
  const GramDims dp = gram_dims(n, k, 1, 256);
  const size_t slices = (size_t)(d.slices > dp.slices ? d.slices : dp.slices) + 1;  // +1: CU counts differ a little
  return ds_align((size_t)n * d.RW * 8) + ds_align(slices * (size_t)n * n * 8) + ds_align((size_t)(n + 1) * d.ld * 8) +
         ds_align((size_t)d.nblk * NB * NB * 8) + 2 * ds_align(panel_bytes(n)) + 2 * ds_align(k * 4) + 2 * ds_align(k * 8) + ds_align(k * 4) +
         ds_align(k * 8) + ds_align(d.RW * 4) * 2 + 4 * ds_align(n * 8) + 8192 +
         ds_align((size_t)((n + 63) / 64) * d.R * 8 + 8) + ds_align((size_t)d.RW * 8 + 8) + ds_align((size_t)d.R * 8 + 8) + 256;
}

// Part 1: everything that does not need the model outputs y (Gram matrix, projection, system matrix).
// It may run on another stream than part 2, concurrently with the masked inference.
int ds_gram_begin(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, int paired, ds_gram_state* gs) {
  hipStream_t st = ctx->stream;
  if (paired && (k & 1)) return ds_fail(ctx, DS_EINVAL, "paired rows need an even row count");
  const int64_t W = (n + 63) / 64;
  const GramDims d = gram_dims(n, k, paired, ctx->num_cus);
  const int64_t R = d.R, RW = d.RW, ld = d.ld;
  gs->n = n; gs->k = k; gs->R = R; gs->RW = RW; gs->ld = ld; gs->nblk = d.nblk; gs->paired = paired;
  gs->Zt = (uint64_t*)ds_arena_alloc(ctx, (size_t)n * RW * 8);
  double* Gp = (double*)ds_arena_alloc(ctx, (size_t)d.slices * n * n * 8);
  gs->M = (double*)ds_arena_alloc(ctx, (size_t)(n + 1) * ld * 8);
  gs->linv = (double*)ds_arena_alloc(ctx, (size_t)d.nblk * NB * NB * 8);
  gs->panel[0] = (double*)ds_arena_alloc(ctx, panel_bytes(n));
  gs->panel[1] = (double*)ds_arena_alloc(ctx, panel_bytes(n));
  float* gw = (float*)ds_arena_alloc(ctx, R * 4);
  float* wu = (float*)ds_arena_alloc(ctx, RW * 4);
  int32_t* uni = (int32_t*)ds_arena_alloc(ctx, RW * 4);
  double* m = (double*)ds_arena_alloc(ctx, n * 8);
  double* stats = (double*)ds_arena_alloc(ctx, 64);
  uint64_t* Zc = (uint64_t*)ds_arena_alloc(ctx, (size_t)W * R * 8 + 8);
  uint64_t* keep = (uint64_t*)ds_arena_alloc(ctx, (size_t)RW * 8 + 8);
  uint64_t* wq = (uint64_t*)ds_arena_alloc(ctx, (size_t)R * 8 + 8);
  double* gscale = (double*)ds_arena_alloc(ctx, 64);
  // buffers of part 2, reserved here so that both parts draw from one contiguous region
  gs->sz = (int32_t*)ds_arena_alloc(ctx, k * 4);
  gs->wc = (float*)ds_arena_alloc(ctx, k * 4);
  gs->t = (double*)ds_arena_alloc(ctx, k * 8);
  gs->sqw = (double*)ds_arena_alloc(ctx, k * 8);
  gs->gc = (double*)ds_arena_alloc(ctx, R * 8);
  gs->c = (double*)ds_arena_alloc(ctx, n * 8);
  gs->yv = (double*)ds_arena_alloc(ctx, n * 8);
  gs->flag = (int*)ds_arena_alloc(ctx, 64);
  if (!gs->Zt || !Gp || !gs->M || !gs->linv || !gs->panel[0] || !gs->panel[1] || !gw || !wu || !uni || !m || !stats || !Zc || !keep || !wq || !gscale || !gs->sz || !gs->wc || !gs->t ||
      !gs->sqw || !gs->gc || !gs->c || !gs->yv || !gs->flag)
    return ds_fail(ctx, DS_EINTERNAL, "gram: arena exhausted");
  hipLaunchKernelGGL(used_row_weights_kernel, dim3(nblocks(R, 256)), dim3(256), 0, st, w, R, paired, gw);
  DS_TRY(ds_bit_transpose(ctx, Z, R, n, W, 0, paired ? 2 : 1, gs->Zt));
  // sparse rows: row-wise outer products into slice 0; the rest (bits in `keep`) column-wise on top of it
  const int64_t row_step = paired ? 2 : 1;
  DS_HIP(ctx, hipMemsetAsync(keep, 0, (size_t)RW * 8, st));
  hipLaunchKernelGGL(gram_scale_kernel, dim3(1), dim3(kThreads), 0, st, gw, R, gscale);
  {
    int64_t blocks = (R * 64 + kThreads - 1) / kThreads;
    if (blocks > (int64_t)ctx->num_cus * 16) blocks = (int64_t)ctx->num_cus * 16;
    hipLaunchKernelGGL(gram_row_class_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, Z, R, W, n, row_step, gw,
                       gscale, sparse_divisor(ctx), Zc, (unsigned long long*)keep, (unsigned long long*)wq);
  }
  hipLaunchKernelGGL(word_weights_kernel, dim3(nblocks(RW, 256)), dim3(256), 0, st, gw, R, RW, Z, W, n, row_step,
                     dense_fraction(ctx), keep, wu, uni);
  const unsigned tiles = nblocks(n, kTile);
  DS_TRY(ds_kernel_mark(ctx, 1, 0));
  hipLaunchKernelGGL(gram_rows_kernel, dim3(tiles, tiles), dim3(kThreads), 0, st, Zc, (const unsigned long long*)wq, R, n,
                     gscale, Gp);
  hipLaunchKernelGGL(gram_kernel, dim3(tiles, tiles, d.slices), dim3(kThreads), 0, st, gs->Zt, n, R, RW, gw, wu, uni, keep,
                     Gp, d.words_per_slice);
  DS_TRY(ds_kernel_mark(ctx, 1, 1));
  const unsigned wblocks = (unsigned)(n < (int64_t)ctx->num_cus * 16 ? n : (int64_t)ctx->num_cus * 16);
  hipLaunchKernelGGL(sum_slices_row_mean_kernel, dim3(wblocks), dim3(kThreads), 0, st, Gp, n, d.slices, m);
  hipLaunchKernelGGL(stats_kernel, dim3(1), dim3(kThreads), 0, st, Gp, m, n, stats);
  hipLaunchKernelGGL(build_matrix_kernel, dim3(nblocks(n * n, 256)), dim3(256), 0, st, Gp, m, stats, n, ld, gs->M,
                     (double*)(gs->flag + 2));
  // the first diagonal block does not involve the right-hand side either: factorised here, off the path that waits
  // for the model outputs
  DS_HIP(ctx, hipMemsetAsync(gs->flag, 0, sizeof(int), st));
  hipLaunchKernelGGL(chol_diag_kernel, dim3(1), dim3(kThreads), 0, st, gs->M, ld, (int64_t)0, (int)(n < NB ? n : NB), gs->linv,
                     gs->flag);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

// Part 2: right-hand side from y, factorisation (the right-hand side rides along as row n), back substitution.
int ds_gram_finish(ds_ctx* ctx, const ds_gram_state* gs, const uint64_t* Z, const float* w, const float* y, float* phi,
                    int defer_check) {
  hipStream_t st = ctx->stream;
  const int64_t n = gs->n, k = gs->k, R = gs->R, RW = gs->RW, ld = gs->ld;
  double* M = gs->M;
  double* linv = gs->linv;
  DS_TRY(ds_row_prep(ctx, Z, k, n, w, y, gs->sz, gs->t, gs->sqw, gs->wc));
  hipLaunchKernelGGL(used_row_rhs_kernel, dim3(nblocks(R, 256)), dim3(256), 0, st, gs->wc, gs->t, R, gs->paired, gs->gc);
  DS_TRY(ds_bit_spmv(ctx, gs->Zt, n, R, RW, 0, 1, gs->gc, gs->c));  // c_j = sum over the rows containing j of gc
  hipLaunchKernelGGL(build_rhs_kernel, dim3(1), dim3(kThreads), 0, st, gs->c, n, ld, M);
  DS_HIP(ctx, hipGetLastError());
  DS_TRY(ds_kernel_mark(ctx, 2, 0));
  const int64_t rows_total = n + 1;  // row n carries the right-hand side
  // While the trailing matrix is large the blocks are taken four at a time (a super-panel of 256 columns):
  // inside it the updates reach only the super-panel's own columns, and the rest of the trailing matrix is
  // updated once with all 256 columns. Below kFuseMaxRows trailing rows: one block per step, the update
  // factorising the next diagonal block on the way.
  bool diag_done = true;  // the first diagonal block was factorised with the system matrix (ds_gram_begin)
  bool panel_ready = false;  // gs->panel[pbuf] holds the rows of the current panel (fused steps only)
  int pbuf = 0;
  int64_t j0 = 0;
  while (j0 < n) {
    const bool super = rows_total - j0 - kSuperCols > kFuseMaxRows && n - j0 >= kSuperCols + NB;
    if (super) {
      for (int b = 0; b < kSuperCols / NB; ++b) {
        const int64_t jb = j0 + (int64_t)b * NB;
        double* li = linv + (size_t)(jb / NB) * NB * NB;
        // inside the super-panel the narrow update factorises the next diagonal block on the way
        if (b == 0 && jb > 0) hipLaunchKernelGGL(chol_diag_kernel, dim3(1), dim3(kThreads), 0, st, M, ld, jb, NB, li, gs->flag);
        const int64_t rest = rows_total - jb - NB;
        const unsigned tt = nblocks(rest, kTile);
        hipLaunchKernelGGL(chol_panel_kernel, dim3(tt), dim3(kThreads), 0, st, M, ld, rows_total, jb, NB, li);
        const unsigned inside = (unsigned)(kSuperCols / NB - 1 - b);  // block columns of the super-panel still ahead
        if (inside > 0)
          hipLaunchKernelGGL(chol_update_kernel<true>, dim3(inside, tt), dim3(kThreads), 0, st, M, ld, rows_total, n, jb,
                             NB, li + (size_t)NB * NB, gs->flag);
      }
      const int64_t base = j0 + kSuperCols;
      const unsigned tw = nblocks(rows_total - base, kTile);
      hipLaunchKernelGGL(chol_update_wide_kernel<(int)kSuperCols>, dim3(tw, tw), dim3(kThreads), 0, st, M, ld, rows_total, n,
                         j0, base);
      j0 += kSuperCols;
      diag_done = false;
      continue;
    }
    const int nb = (int)(n - j0 < NB ? n - j0 : NB);
    double* li = linv + (size_t)(j0 / NB) * NB * NB;
    // a diagonal block has a launch of its own only if the update before it did not factorise it already
    if (!diag_done) hipLaunchKernelGGL(chol_diag_kernel, dim3(1), dim3(kThreads), 0, st, M, ld, j0, nb, li, gs->flag);
    diag_done = false;
    const int64_t rest = rows_total - j0 - nb;
    if (n - j0 - nb > 0 && rest <= kFuseMaxRows) {  // nb == NB here
      const unsigned tt = nblocks(rest, kTile);
      if (!panel_ready) {
        hipLaunchKernelGGL(copy_panel_kernel, dim3(nblocks(rest * NB, 256)), dim3(256), 0, st, M, ld, rows_total, j0 + NB, j0, n,
                           gs->panel[pbuf]);
        panel_ready = true;
      }
      hipLaunchKernelGGL(chol_step_kernel, dim3(tt, tt), dim3(kThreads), 0, st, M, ld, rows_total, n, j0, li,
                         li + (size_t)NB * NB, gs->flag, gs->panel[pbuf], gs->panel[pbuf ^ 1]);
      pbuf ^= 1;
      diag_done = true;
      j0 += nb;
      continue;
    }
    hipLaunchKernelGGL(chol_panel_kernel, dim3(nblocks(rest, kTile)), dim3(kThreads), 0, st, M, ld, rows_total, j0, nb, li);
    if (n - j0 - nb > 0) {
      const unsigned tt = nblocks(rest, kTile);
      if (rest <= kFuseMaxRows) {
        hipLaunchKernelGGL(chol_update_kernel<true>, dim3(tt, tt), dim3(kThreads), 0, st, M, ld, rows_total, n, j0, nb,
                           li + (size_t)NB * NB, gs->flag);
        diag_done = true;
      } else {
        hipLaunchKernelGGL(chol_update_kernel<false>, dim3(tt, tt), dim3(kThreads), 0, st, M, ld, rows_total, n, j0, nb,
                           (double*)nullptr, gs->flag);
      }
    }
    j0 += nb;
  }
  DS_TRY(ds_kernel_mark(ctx, 2, 1));
  if (n <= kBackSmallMax) {
    hipLaunchKernelGGL(chol_back_small_kernel, dim3(1), dim3(kBackThreads), 0, st, M, ld, n, (int)gs->nblk, linv, y, phi);
  } else {
  hipLaunchKernelGGL(copy_row_kernel, dim3(nblocks(n, 256)), dim3(256), 0, st, M, ld, n, gs->yv);
  for (int64_t bk = gs->nblk - 1; bk >= 0; --bk) {
    const int64_t j0 = bk * NB;
    const int nb = (int)(n - j0 < NB ? n - j0 : NB);
    const unsigned wgs = j0 > 0 ? nblocks(j0, kThreads) : 1;
    hipLaunchKernelGGL(chol_back_step_kernel, dim3(wgs), dim3(kThreads), 0, st, M, ld, j0, nb,
                       linv + (size_t)bk * NB * NB, gs->yv, gs->c);  // c is free again: it receives psi
  }
  hipLaunchKernelGGL(finish_phi_kernel, dim3(nblocks(n, 256)), dim3(256), 0, st, gs->c, y, n, phi);
  }
  DS_HIP(ctx, hipGetLastError());
  if (defer_check) return DS_OK;  // the caller reads gs->flag back with its own results
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail, gs->flag, sizeof(int), hipMemcpyDeviceToHost, st));
  DS_HIP(ctx, hipStreamSynchronize(st));
  if (*(int*)ctx->h_mail != 0)
    return ds_fail(ctx, DS_ESINGULAR, "Cholesky met a non-positive pivot: the sampled rows do not determine all %lld players", (long long)n);
  return DS_OK;
}

int ds_solve_gram_chol(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, const float* y, int paired,
                       float* phi) {
  ds_gram_state gs;
  DS_TRY(ds_gram_begin(ctx, n, k, Z, w, paired, &gs));
  return ds_gram_finish(ctx, &gs, Z, w, y, phi, 0);
}
