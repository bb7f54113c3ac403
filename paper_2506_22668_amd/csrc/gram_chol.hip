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
// a word that straddles weight classes walks the set bits of the AND.
#include "internal.h"
#include "solve_common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kTile = 64;
constexpr int kChunk = 32;  // 64-row words per LDS chunk

// per word of 64 rows: the common weight, or non-uniform
__global__ void word_weights_kernel(const float* w, int64_t k, int64_t KW, float* wu, int32_t* uni) {
  const int64_t wd = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (wd >= KW) return;
  const int64_t i0 = wd * 64;
  const float first = w[i0];
  int same = 1;
  for (int b = 1; b < 64; ++b) {
    const int64_t i = i0 + b;
    if (i < k && w[i] != first) same = 0;
  }
  wu[wd] = first;
  uni[wd] = same;
}

__global__ __launch_bounds__(kThreads) void gram_kernel(const uint64_t* Zt, int64_t n, int64_t k, int64_t KW,
                                                        const float* w, const float* wu, const int32_t* uni, double* G) {
  const int ta = blockIdx.y, tb = blockIdx.x;
  if (tb > ta) return;
  __shared__ uint64_t As[kTile][kChunk + 1];
  __shared__ uint64_t Bs[kTile][kChunk + 1];
  __shared__ float wrow[kChunk * 64];
  __shared__ float wus[kChunk];
  __shared__ int unis[kChunk];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int64_t a0 = (int64_t)ta * kTile, b0 = (int64_t)tb * kTile;
  double acc[4][4];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
  for (int64_t wd0 = 0; wd0 < KW; wd0 += kChunk) {
    __syncthreads();
    for (int idx = tid; idx < kTile * kChunk; idx += kThreads) {
      const int r = idx / kChunk, c = idx - r * kChunk;
      const int64_t wd = wd0 + c;
      As[r][c] = (a0 + r < n && wd < KW) ? Zt[(a0 + r) * KW + wd] : 0ull;
      Bs[r][c] = (b0 + r < n && wd < KW) ? Zt[(b0 + r) * KW + wd] : 0ull;
    }
    for (int idx = tid; idx < kChunk * 64; idx += kThreads) {
      const int64_t i = wd0 * 64 + idx;
      wrow[idx] = i < k ? w[i] : 0.f;
    }
    if (tid < kChunk) {
      const int64_t wd = wd0 + tid;
      wus[tid] = wd < KW ? wu[wd] : 0.f;
      unis[tid] = wd < KW ? uni[wd] : 1;
    }
    __syncthreads();
    float f[4][4];
    for (int i = 0; i < 4; ++i)
      for (int j = 0; j < 4; ++j) f[i][j] = 0.f;
    for (int c = 0; c < kChunk; ++c) {
      uint64_t av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        av[i] = As[ty + 16 * i][c];
        bv[i] = Bs[tx + 16 * i][c];
      }
      if (unis[c]) {
        const float wv = wus[c];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) f[i][j] += wv * (float)__popcll(av[i] & bv[j]);
      } else {
        const float* wr = wrow + c * 64;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            uint64_t m = av[i] & bv[j];
            float s = 0.f;
            while (m) {
              s += wr[__ffsll((long long)m) - 1];
              m &= m - 1;
            }
            f[i][j] += s;
          }
      }
    }
    for (int i = 0; i < 4; ++i)
      for (int j = 0; j < 4; ++j) acc[i][j] += (double)f[i][j];
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      const int64_t a = a0 + ty + 16 * i, b = b0 + tx + 16 * j;
      if (a < n && b < n) {
        G[a * n + b] = acc[i][j];
        G[b * n + a] = acc[i][j];
      }
    }
}

// c_j = sum_i w_i t_i z_ij, one wave per column of the transposed matrix
__global__ __launch_bounds__(kThreads) void rhs_kernel(const uint64_t* Zt, int64_t n, int64_t k, int64_t KW,
                                                       const float* w, const double* t, double* c) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t j = wave; j < n; j += nwaves) {
    double s = 0.0;
    for (int64_t wd = 0; wd < KW; ++wd) {
      const uint64_t word = Zt[j * KW + wd];
      const int64_t i = wd * 64 + lane;
      if (i < k && ((word >> lane) & 1ull)) s += (double)w[i] * t[i];
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) c[j] = s;
  }
}

// row means of G
__global__ __launch_bounds__(kThreads) void row_mean_kernel(const double* G, int64_t n, double* m) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t a = wave; a < n; a += nwaves) {
    double s = 0.0;
    for (int64_t b = lane; b < n; b += 64) s += G[a * n + b];
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) m[a] = s / (double)n;
  }
}

// single block: stats[0] = mu (grand mean), stats[1] = trace(G), stats[2] = mean(c)
__global__ __launch_bounds__(kThreads) void stats_kernel(const double* G, const double* m, const double* c, int64_t n,
                                                         double* stats) {
  __shared__ double sh[3][kThreads];
  double a = 0, b = 0, d = 0;
  for (int64_t i = threadIdx.x; i < n; i += kThreads) {
    a += m[i];
    b += G[i * n + i];
    d += c[i];
  }
  sh[0][threadIdx.x] = a;
  sh[1][threadIdx.x] = b;
  sh[2][threadIdx.x] = d;
  __syncthreads();
  if (threadIdx.x == 0) {
    double x = 0, yv = 0, z = 0;
    for (int i = 0; i < kThreads; ++i) {
      x += sh[0][i];
      yv += sh[1][i];
      z += sh[2][i];
    }
    stats[0] = x / (double)n;
    stats[1] = yv;
    stats[2] = z / (double)n;
  }
}

// A = P G P + gamma 11^T / n in place; rhs = c - mean(c). gamma = trace(PGP)/(n-1).
__global__ void build_system_kernel(double* G, const double* m, double* c, const double* stats, int64_t n) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const double mu = stats[0];
  const double tr = stats[1] - (double)n * mu;
  double gamma = tr / (double)(n > 1 ? n - 1 : 1);
  if (!(gamma > 0.0)) gamma = 1.0;
  if (idx < n * n) {
    const int64_t a = idx / n, b = idx - a * n;
    G[idx] = G[idx] - m[a] - m[b] + mu + gamma / (double)n;
  }
  if (idx < n) c[idx] -= stats[2];
}

// ---------------- blocked Cholesky (lower, in place, fp64) ----------------
constexpr int NB = 64;

__global__ __launch_bounds__(kThreads) void chol_diag_kernel(double* A, int64_t n, int64_t j0, int nb, int* flag) {
  __shared__ double S[NB][NB + 1];
  for (int idx = threadIdx.x; idx < NB * NB; idx += kThreads) {
    const int r = idx / NB, c = idx - r * NB;
    S[r][c] = (r < nb && c < nb) ? A[(j0 + r) * n + j0 + c] : (r == c ? 1.0 : 0.0);
  }
  __syncthreads();
  for (int kk = 0; kk < nb; ++kk) {
    if (threadIdx.x == 0) {
      double p = S[kk][kk];
      if (!(p > 0.0)) {
        atomicExch(flag, 1);
        p = 1.0;
      }
      S[kk][kk] = sqrt(p);
    }
    __syncthreads();
    const double d = S[kk][kk];
    for (int r = kk + 1 + threadIdx.x; r < nb; r += kThreads) S[r][kk] /= d;
    __syncthreads();
    const int rem = nb - kk - 1;
    for (int idx = threadIdx.x; idx < rem * rem; idx += kThreads) {
      const int r = kk + 1 + idx / rem, c = kk + 1 + idx % rem;
      if (c <= r) S[r][c] -= S[r][kk] * S[c][kk];
    }
    __syncthreads();
  }
  for (int idx = threadIdx.x; idx < NB * NB; idx += kThreads) {
    const int r = idx / NB, c = idx - r * NB;
    if (r < nb && c <= r) A[(j0 + r) * n + j0 + c] = S[r][c];
  }
}

// rows below the diagonal block: X L11^T = A21, one thread per row
__global__ __launch_bounds__(64) void chol_panel_kernel(double* A, int64_t n, int64_t j0, int nb) {
  __shared__ double Ls[NB][NB + 1];
  for (int idx = threadIdx.x; idx < NB * NB; idx += 64) {
    const int r = idx / NB, c = idx - r * NB;
    Ls[r][c] = (r < nb && c <= r) ? A[(j0 + r) * n + j0 + c] : (r == c ? 1.0 : 0.0);
  }
  __syncthreads();
  const int64_t i = j0 + nb + (int64_t)blockIdx.x * 64 + threadIdx.x;
  if (i >= n) return;
  double x[NB];
#pragma unroll
  for (int c = 0; c < NB; ++c) x[c] = c < nb ? A[i * n + j0 + c] : 0.0;
#pragma unroll
  for (int c = 0; c < NB; ++c) {
    double v = x[c];
#pragma unroll
    for (int m = 0; m < c; ++m) v -= x[m] * Ls[c][m];
    x[c] = v / Ls[c][c];
  }
#pragma unroll
  for (int c = 0; c < NB; ++c)
    if (c < nb) A[i * n + j0 + c] = x[c];
}

// trailing update A22 -= L21 L21^T on the lower tiles
__global__ __launch_bounds__(kThreads) void chol_update_kernel(double* A, int64_t n, int64_t j0, int nb) {
  const int ti = blockIdx.y, tj = blockIdx.x;
  if (tj > ti) return;
  __shared__ double Li[kTile][NB + 1];
  __shared__ double Lj[kTile][NB + 1];
  const int64_t base = j0 + nb;
  const int64_t i0 = base + (int64_t)ti * kTile, c0 = base + (int64_t)tj * kTile;
  for (int idx = threadIdx.x; idx < kTile * NB; idx += kThreads) {
    const int r = idx / NB, c = idx - r * NB;
    Li[r][c] = (i0 + r < n && c < nb) ? A[(i0 + r) * n + j0 + c] : 0.0;
    Lj[r][c] = (c0 + r < n && c < nb) ? A[(c0 + r) * n + j0 + c] : 0.0;
  }
  __syncthreads();
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  double acc[4][4];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
  for (int m = 0; m < NB; ++m) {
    double a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[i] = Li[ty + 16 * i][m];
      b[i] = Lj[tx + 16 * i][m];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      const int64_t r = i0 + ty + 16 * i, c = c0 + tx + 16 * j;
      if (r < n && c <= r) A[r * n + c] -= acc[i][j];
    }
}

// L y = b then L^T x = y, single workgroup, blocked by NB; b is overwritten by x.
__global__ __launch_bounds__(kThreads) void chol_solve_kernel(const double* A, int64_t n, double* b) {
  __shared__ double Ls[NB][NB + 1];
  __shared__ double xs[NB];
  const int tid = threadIdx.x;
  // forward
  for (int64_t j0 = 0; j0 < n; j0 += NB) {
    const int nb = (int)(n - j0 < NB ? n - j0 : NB);
    for (int idx = tid; idx < NB * NB; idx += kThreads) {
      const int r = idx / NB, c = idx - r * NB;
      Ls[r][c] = (r < nb && c <= r) ? A[(j0 + r) * n + j0 + c] : (r == c ? 1.0 : 0.0);
    }
    __syncthreads();
    if (tid < 64) {
      double v = tid < nb ? b[j0 + tid] : 0.0;
      for (int c = 0; c < nb; ++c) {
        const double piv = __shfl(v, c, 64) / Ls[c][c];
        if (tid == c) v = piv;
        if (tid > c) v -= Ls[tid][c] * piv;
      }
      xs[tid] = v;
      if (tid < nb) b[j0 + tid] = v;
    }
    __syncthreads();
    for (int64_t i = j0 + nb + tid; i < n; i += kThreads) {
      double s = 0.0;
      for (int c = 0; c < nb; ++c) s += A[i * n + j0 + c] * xs[c];
      b[i] -= s;
    }
    __syncthreads();
  }
  // backward
  const int64_t nblk = (n + NB - 1) / NB;
  for (int64_t bk = nblk - 1; bk >= 0; --bk) {
    const int64_t j0 = bk * NB;
    const int nb = (int)(n - j0 < NB ? n - j0 : NB);
    for (int idx = tid; idx < NB * NB; idx += kThreads) {
      const int r = idx / NB, c = idx - r * NB;
      Ls[r][c] = (r < nb && c <= r) ? A[(j0 + r) * n + j0 + c] : (r == c ? 1.0 : 0.0);
    }
    __syncthreads();
    if (tid < 64) {
      double v = tid < nb ? b[j0 + tid] : 0.0;
      for (int c = nb - 1; c >= 0; --c) {
        const double piv = __shfl(v, c, 64) / Ls[c][c];
        if (tid == c) v = piv;
        if (tid < c) v -= Ls[c][tid] * piv;
      }
      xs[tid] = v;
      if (tid < nb) b[j0 + tid] = v;
    }
    __syncthreads();
    for (int64_t j = tid; j < j0; j += kThreads) {
      double s = 0.0;
      for (int r = 0; r < nb; ++r) s += A[(j0 + r) * n + j] * xs[r];
      b[j] -= s;
    }
    __syncthreads();
  }
}

__global__ void finish_phi_kernel(const double* psi, const float* y, int64_t n, float* phi) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const double delta = (double)y[1] - (double)y[0];
  phi[j] = (float)(psi[j] + delta / (double)n);
}

inline unsigned nblocks(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

size_t ds_gram_arena_bytes(int64_t n, int64_t k) {
  const int64_t KW = (k + 63) / 64;
  return ds_align((size_t)n * KW * 8) + ds_align((size_t)n * n * 8) + 2 * ds_align(k * 4) + 2 * ds_align(k * 8) +
         ds_align(KW * 4) * 2 + 3 * ds_align(n * 8) + 4096;
}

int ds_solve_gram_chol(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, const float* y, float* phi) {
  hipStream_t st = ctx->stream;
  const int64_t KW = (k + 63) / 64, W = (n + 63) / 64;
  uint64_t* Zt = (uint64_t*)ds_arena_alloc(ctx, (size_t)n * KW * 8);
  double* G = (double*)ds_arena_alloc(ctx, (size_t)n * n * 8);
  int32_t* sz = (int32_t*)ds_arena_alloc(ctx, k * 4);
  float* wc = (float*)ds_arena_alloc(ctx, k * 4);
  double* t = (double*)ds_arena_alloc(ctx, k * 8);
  double* sqw = (double*)ds_arena_alloc(ctx, k * 8);
  float* wu = (float*)ds_arena_alloc(ctx, KW * 4);
  int32_t* uni = (int32_t*)ds_arena_alloc(ctx, KW * 4);
  double* c = (double*)ds_arena_alloc(ctx, n * 8);
  double* m = (double*)ds_arena_alloc(ctx, n * 8);
  double* stats = (double*)ds_arena_alloc(ctx, 64);
  int* flag = (int*)ds_arena_alloc(ctx, 64);
  if (!Zt || !G || !sz || !wc || !t || !sqw || !wu || !uni || !c || !m || !stats || !flag)
    return ds_fail(ctx, DS_EINTERNAL, "gram: arena exhausted");
  DS_HIP(ctx, hipMemsetAsync(flag, 0, sizeof(int), st));
  DS_TRY(ds_row_prep(ctx, Z, k, n, w, y, sz, t, sqw, wc));
  DS_TRY(ds_bit_transpose(ctx, Z, k, n, W, 0, 1, Zt));
  hipLaunchKernelGGL(word_weights_kernel, dim3(nblocks(KW, 256)), dim3(256), 0, st, wc, k, KW, wu, uni);
  const unsigned tiles = nblocks(n, kTile);
  DS_TRY(ds_kernel_mark(ctx, 1, 0));
  hipLaunchKernelGGL(gram_kernel, dim3(tiles, tiles), dim3(kThreads), 0, st, Zt, n, k, KW, wc, wu, uni, G);
  DS_TRY(ds_kernel_mark(ctx, 1, 1));
  const unsigned wblocks = (unsigned)(((n * 64 + kThreads - 1) / kThreads) < (int64_t)ctx->num_cus * 8 ? ((n * 64 + kThreads - 1) / kThreads) : (int64_t)ctx->num_cus * 8);
  hipLaunchKernelGGL(rhs_kernel, dim3(wblocks), dim3(kThreads), 0, st, Zt, n, k, KW, wc, t, c);
  hipLaunchKernelGGL(row_mean_kernel, dim3(wblocks), dim3(kThreads), 0, st, G, n, m);
  hipLaunchKernelGGL(stats_kernel, dim3(1), dim3(kThreads), 0, st, G, m, c, n, stats);
  hipLaunchKernelGGL(build_system_kernel, dim3(nblocks(n * n, 256)), dim3(256), 0, st, G, m, c, stats, n);
  DS_HIP(ctx, hipGetLastError());
  DS_TRY(ds_kernel_mark(ctx, 2, 0));
  for (int64_t j0 = 0; j0 < n; j0 += NB) {
    const int nb = (int)(n - j0 < NB ? n - j0 : NB);
    hipLaunchKernelGGL(chol_diag_kernel, dim3(1), dim3(kThreads), 0, st, G, n, j0, nb, flag);
    const int64_t rest = n - j0 - nb;
    if (rest > 0) {
      hipLaunchKernelGGL(chol_panel_kernel, dim3(nblocks(rest, 64)), dim3(64), 0, st, G, n, j0, nb);
      const unsigned tt = nblocks(rest, kTile);
      hipLaunchKernelGGL(chol_update_kernel, dim3(tt, tt), dim3(kThreads), 0, st, G, n, j0, nb);
    }
  }
  DS_TRY(ds_kernel_mark(ctx, 2, 1));
  hipLaunchKernelGGL(chol_solve_kernel, dim3(1), dim3(kThreads), 0, st, G, n, c);
  hipLaunchKernelGGL(finish_phi_kernel, dim3(nblocks(n, 256)), dim3(256), 0, st, c, y, n, phi);
  DS_HIP(ctx, hipGetLastError());
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail, flag, sizeof(int), hipMemcpyDeviceToHost, st));
  DS_HIP(ctx, hipStreamSynchronize(st));
  if (*(int*)ctx->h_mail != 0)
    return ds_fail(ctx, DS_ESINGULAR, "Cholesky met a non-positive pivot: the sampled rows do not determine all %lld players", (long long)n);
  return DS_OK;
}
