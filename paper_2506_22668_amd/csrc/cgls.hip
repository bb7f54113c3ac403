// Conjugate gradients for least squares on the bit-packed mask matrix.
//
// Paper, Alg. 1 (CGLS on sqrt(W) M with a 1D row layout; here one GPU holds all
// rows, so the two all-reduces of the algorithm are plain device reductions). The
// iteration is the standard Hestenes-Stiefel form (the step ratio is
// |s_i|^2/|s_(i-1)|^2), started from zero, on the matrix sqrt(W) Z P with
// P = I - 11^T/n, so the iterate stays orthogonal to 1 and, when the problem is
// rank-deficient, converges to the minimum-norm solution.
//
// Both products walk set bits only. With complementary pairs (rows 2r, 2r+1 with
// one weight) only the small member of each pair is read:
//   forward:  d_r = sum_{j in S_r} u_j;  v_2r = a_r d_r,  v_2r+1 = a_r (sum(u) - d_r)
//   adjoint:  s = P sum_r a_r (r_2r - r_2r+1) z_r          (constants vanish under P)
// and the adjoint runs the same row kernel on a transposed copy of the small rows.
// Without the pairing promise every row is walked and the transpose holds all rows.
// All vectors and sums are fp64 (fp64 adds run at the rate of unpacked fp32 here).
#include "internal.h"
#include "solve_common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kRed = 1024;  // blocks (and partials) of every reduction, at most

__device__ __forceinline__ void block_reduce2(double a, double b, double* pa, double* pb) {
  __shared__ double sh[2][kThreads / 64];
  for (int o = 32; o > 0; o >>= 1) {
    a += __shfl_xor(a, o, 64);
    b += __shfl_xor(b, o, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    sh[0][threadIdx.x >> 6] = a;
    sh[1][threadIdx.x >> 6] = b;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double x = 0, y = 0;
    for (int i = 0; i < kThreads / 64; ++i) {
      x += sh[0][i];
      y += sh[1][i];
    }
    *pa = x;
    *pb = y;
  }
  __syncthreads();
}

// scalars (device doubles): 0 gamma, 1 delta, 2 theta, 3 beta, 4 sum(u), 5 mean(s_raw), 6 gamma_new, 7 gamma0,
// 8 done (0/1), 9 iterations completed, 10 relative residual at the last test
// partial sums: four arrays of kRed doubles, one per reduction of the loop (|v|^2, sum(s), |Ps|^2, sum(u)), so
// that a kernel can read the partials of the reduction before it while writing those of its own
struct Vecs {
  int64_t n, k, R;   // R = rows of the forward matrix (pairs or rows)
  int paired;
  const double* sqw; // [k]
  double *x, *u, *s, *r, *v, *d, *h;  // n, n, n, k, k, R, R
  double* scal;
  double* part;      // [4 * kRed]
  // fixed-point products only (else null): where the kernel that writes u (h) leaves the bit pattern of max |u| (max |h|)
  // for the next forward (adjoint) product, which then needs no pass of its own over the vector
  unsigned long long *slot_u, *slot_h;
  // fixed-point products inside the loop (fused != 0): the products leave their integer partial sums, and the loop's
  // kernel that reads d (s) first adds them up itself, scales them by scal_f[0] (scal_a[0]) and clears the product's
  // maximum slot. Forward: the rows [0, Rs) come from the tiles, the rest from the matrix cores; adjoint: both parts
  // cover all n entries and are added, tiles first.
  int fused;
  int64_t Rs;
  ds_fixed_view fwd, adj;
  const double *scal_f, *scal_a;
};

// T lanes (a power of two, consecutive lanes of a wave, `sub` = the lane's place among them) add up one entry together:
// each takes every T-th group, the integers are added across the lanes, and all T lanes return the same value
template <int T>
__device__ __forceinline__ double mm_result(const ds_fixed_view& v, int64_t r, int sub) {
  long long S[7] = {0, 0, 0, 0, 0, 0, 0};
  ds_mm_sum_part(v.mm_partial, v.mm_rows, v.mm_groups, r, sub, T, S);
#pragma unroll
  for (int o = 1; o < T; o <<= 1)
#pragma unroll
    for (int d = 0; d < 7; ++d) S[d] += __shfl_xor(S[d], o, 64);
  return ds_mm_sum_finish(S);
}
template <int T>
__device__ __forceinline__ double tile_result(const ds_fixed_view& v, int64_t i, int sub) {
  long long hi = 0, lo = 0;
  ds_tile_sum_part(v.tile_partial, v.tile_len, v.tile_groups, i, sub, T, hi, lo);
#pragma unroll
  for (int o = 1; o < T; o <<= 1) {
    hi += __shfl_xor(hi, o, 64);
    lo += __shfl_xor(lo, o, 64);
  }
  return ds_tile_sum_finish(hi, lo, v.tile_sh);
}
template <int T>
__device__ __forceinline__ double forward_result(const Vecs& a, double sc, int64_t i, int sub) {
  if (i < a.Rs) return a.fwd.tile_groups ? tile_result<T>(a.fwd, i, sub) * sc : 0.0;
  return mm_result<T>(a.fwd, i - a.Rs, sub) * sc;
}
template <int T>
__device__ __forceinline__ double adjoint_result(const Vecs& a, double sc, int64_t j, int sub) {
  const double mm = a.adj.mm_groups ? mm_result<T>(a.adj, j, sub) * sc : 0.0;
  if (!a.adj.tile_groups) return mm;
  const double tl = tile_result<T>(a.adj, j, sub) * sc;
  return a.adj.mm_groups ? tl + mm : tl;
}

// the workgroup's part of max |x| (bit patterns of non-negative doubles order like the values) into *slot
// (one atomic per workgroup: every thread of the workgroup must call this)
__device__ __forceinline__ void publish_absmax(unsigned long long m, unsigned long long* slot) {
  __shared__ unsigned long long wm[kThreads / 64];
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long t = __shfl_xor(m, o, 64);
    m = t > m ? t : m;
  }
  if ((threadIdx.x & 63) == 0) wm[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < kThreads / 64; ++i) m = wm[i] > m ? wm[i] : m;
    if (m) atomicMax(slot, m);
  }
  __syncthreads();
}
__device__ __forceinline__ unsigned long long abs_bits(double x) {
  return (unsigned long long)__double_as_longlong(x) & 0x7fffffffffffffffull;
}
// (an iteration that has stopped leaves the vector alone, but the products queued behind it still read its maximum)
__device__ __forceinline__ void publish_absmax_of(const double* x, int64_t len, unsigned long long* slot) {
  if (!slot) return;
  unsigned long long m = 0;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < len; i += (int64_t)gridDim.x * kThreads) {
    const unsigned long long b = abs_bits(x[i]);
    m = b > m ? b : m;
  }
  publish_absmax(m, slot);
}

// r = sqrt(w) t ; h from r
__global__ void init_r_kernel(Vecs a, const double* t) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < a.k) a.r[i] = a.sqw[i] * t[i];
}
__global__ void make_h_kernel(Vecs a) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= a.R) return;
  a.h[i] = a.paired ? a.sqw[2 * i] * (a.r[2 * i] - a.r[2 * i + 1]) : a.sqw[i] * a.r[i];
}

// sum of nparts (<= kRed) partials by one wave, in a fixed order; every lane gets the result
__device__ __forceinline__ double wave_sum_partials(const double* part, int nparts) {
  double s = 0.0;
  for (int i = threadIdx.x; i < nparts; i += 64) s += part[i];
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  return s;
}

// partial sums of the raw adjoint (for its mean)
__global__ __launch_bounds__(kThreads) void s_sum_kernel(Vecs a) {
  double s1 = 0;
  for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < a.n; j += (int64_t)gridDim.x * kThreads) s1 += a.s[j];
  double dummy;
  block_reduce2(s1, 0.0, &a.part[blockIdx.x], &dummy);
}

__global__ void fin_mean_kernel(Vecs a, int nparts) {
  const double s1 = wave_sum_partials(a.part, nparts);
  if (threadIdx.x == 0) a.scal[5] = s1 / (double)a.n;
}

// s <- P s (subtract the mean in place) and partial |P s|^2. Two passes on purpose:
// the raw adjoint carries a large common offset, and sum(s^2) - n mean^2 would cancel.
__global__ __launch_bounds__(kThreads) void s_center_kernel(Vecs a) {
  const double mean = a.scal[5];
  double s2 = 0;
  for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < a.n; j += (int64_t)gridDim.x * kThreads) {
    const double v = a.s[j] - mean;
    a.s[j] = v;
    s2 += v * v;
  }
  double dummy;
  block_reduce2(s2, 0.0, &a.part[blockIdx.x], &dummy);
}

// gamma_new = |P s|^2 and beta; the first call sets gamma0 and beta = theta = 0
__global__ void fin_gamma_kernel(Vecs a, int nparts, int first) {
  const double g = wave_sum_partials(a.part, nparts);
  if (threadIdx.x != 0) return;
  a.scal[6] = g;
  if (first) {
    a.scal[7] = g;
    a.scal[3] = 0.0;
    a.scal[2] = 0.0;
  } else {
    a.scal[3] = a.scal[0] > 0.0 ? g / a.scal[0] : 0.0;
  }
}

// x += theta u ; u = s + beta u (s already projected) ; partial sum(u)
__global__ __launch_bounds__(kThreads) void update_xu_kernel(Vecs a) {
  const double th = a.scal[2], beta = a.scal[3];
  double acc = 0;
  for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < a.n; j += (int64_t)gridDim.x * kThreads) {
    const double uo = a.u[j];
    a.x[j] += th * uo;
    const double un = a.s[j] + beta * uo;
    a.u[j] = un;
    acc += un;
  }
  double dummy;
  block_reduce2(acc, 0.0, &a.part[blockIdx.x], &dummy);
}

__global__ void fin_u_kernel(Vecs a, int nparts) {
  const double s = wave_sum_partials(a.part, nparts);
  if (threadIdx.x == 0) {
    a.scal[4] = s;
    a.scal[0] = a.scal[6];
  }
}

// ---- the loop's kernels: every reduction is finished by the kernel that needs its result (each workgroup
// adds the same partials in the same order, workgroup 0 records the scalar), and the stopping rule of the
// iteration is evaluated on the device, so that the host only looks every few iterations. Once `done` is set
// the state that the result is made of (x, u, theta) is left alone by everything that still runs. ----
constexpr int kPartV = 0, kPartS = 1, kPartG = 2, kPartU = 3;

// all threads of the workgroup get the sum of the nparts partials of array `which`
// (every workgroup adds them in the same order: thread t takes the partials t, t + kThreads, ..., then lanes, then waves)
__device__ __forceinline__ double block_sum_partials(const Vecs& a, int which, int nparts) {
  __shared__ double bs[kThreads / 64];
  const double* part = a.part + which * kRed;
  double s = 0.0;
  for (int i = threadIdx.x; i < nparts; i += kThreads) s += part[i];
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) bs[threadIdx.x >> 6] = s;
  __syncthreads();
  double t = bs[0];
  for (int i = 1; i < kThreads / 64; ++i) t += bs[i];
  return t;
}

// v from d (after finishing sum(u) and moving gamma_new to gamma); partial |v|^2. T lanes per row (1 unless fused).
template <int T>
__global__ __launch_bounds__(kThreads) void loop_make_v_kernel(Vecs a, int parts_u) {
  const double U = block_sum_partials(a, kPartU, parts_u);
  if (blockIdx.x == 0 && threadIdx.x == 0 && a.scal[8] == 0.0) {
    a.scal[4] = U;
    a.scal[0] = a.scal[6];
  }
  const double sc = a.fused ? a.scal_f[0] : 0.0;
  if (a.fused && blockIdx.x == 0 && threadIdx.x == 0) *a.slot_u = 0ull;
  double acc = 0.0;
  const int sub = threadIdx.x & (T - 1);
  for (int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / T; i < a.R; i += (int64_t)gridDim.x * (kThreads / T)) {
    const double d = a.fused ? forward_result<T>(a, sc, i, sub) : a.d[i];
    if (sub == 0) {   // (all T lanes hold the same d)
      if (a.paired) {
        const double w = a.sqw[2 * i];
        const double v0 = w * d, v1 = w * (U - d);
        a.v[2 * i] = v0;
        a.v[2 * i + 1] = v1;
        acc += v0 * v0 + v1 * v1;
      } else {
        const double v0 = a.sqw[i] * d;
        a.v[i] = v0;
        acc += v0 * v0;
      }
    }
  }
  double dummy;
  block_reduce2(acc, 0.0, &a.part[kPartV * kRed + blockIdx.x], &dummy);
}

// delta = |v|^2, theta = gamma / delta; r -= theta v, then h. A direction in the null space (delta = 0)
// ends the iteration with theta = 0.
__global__ __launch_bounds__(kThreads) void loop_update_r_kernel(Vecs a, int parts_v) {
  const double delta = block_sum_partials(a, kPartV, parts_v);
  const bool done = a.scal[8] != 0.0;
  const double gamma = a.scal[0];
  const bool null_dir = !(delta > 0.0);
  const double th = null_dir ? 0.0 : gamma / delta;
  if (done) {
    publish_absmax_of(a.h, a.R, a.slot_h);
    return;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    a.scal[1] = delta;
    a.scal[2] = th;
    if (null_dir) {
      a.scal[8] = 1.0;
      a.scal[9] += 1.0;
    }
  }
  unsigned long long hm = 0;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < a.R; i += (int64_t)gridDim.x * kThreads) {
    double hn;
    if (a.paired) {
      const double r0 = a.r[2 * i] - th * a.v[2 * i], r1 = a.r[2 * i + 1] - th * a.v[2 * i + 1];
      a.r[2 * i] = r0;
      a.r[2 * i + 1] = r1;
      hn = a.sqw[2 * i] * (r0 - r1);
    } else {
      const double r0 = a.r[i] - th * a.v[i];
      a.r[i] = r0;
      hn = a.sqw[i] * r0;
    }
    a.h[i] = hn;
    const unsigned long long b = abs_bits(hn);
    hm = b > hm ? b : hm;
  }
  if (a.slot_h) publish_absmax(hm, a.slot_h);
}

template <int T>
__global__ __launch_bounds__(kThreads) void loop_s_sum_kernel(Vecs a) {
  double s1 = 0;
  if (a.fused) {
    const double sc = a.scal_a[0];
    if (blockIdx.x == 0 && threadIdx.x == 0) *a.slot_h = 0ull;
    const int sub = threadIdx.x & (T - 1);
    for (int64_t j = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / T; j < a.n; j += (int64_t)gridDim.x * (kThreads / T)) {
      const double v = adjoint_result<T>(a, sc, j, sub);
      if (sub == 0) {
        a.s[j] = v;
        s1 += v;
      }
    }
  } else {
    for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < a.n; j += (int64_t)gridDim.x * kThreads) s1 += a.s[j];
  }
  double dummy;
  block_reduce2(s1, 0.0, &a.part[kPartS * kRed + blockIdx.x], &dummy);
}

// s <- P s and partial |P s|^2 (two passes on purpose, see s_center_kernel)
__global__ __launch_bounds__(kThreads) void loop_s_center_kernel(Vecs a, int parts_s) {
  const double mean = block_sum_partials(a, kPartS, parts_s) / (double)a.n;
  double s2 = 0;
  for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < a.n; j += (int64_t)gridDim.x * kThreads) {
    const double v = a.s[j] - mean;
    a.s[j] = v;
    s2 += v * v;
  }
  double dummy;
  block_reduce2(s2, 0.0, &a.part[kPartG * kRed + blockIdx.x], &dummy);
}

// end of an iteration: gamma_new = |P s|^2, the stopping rule, and (if the iteration goes on and do_update)
// x += theta u, u = s + beta u with the partial sums of the new u
__global__ __launch_bounds__(kThreads) void loop_update_xu_kernel(Vecs a, int parts_g, double tol, int do_update) {
  const double g = block_sum_partials(a, kPartG, parts_g);
  if (a.scal[8] != 0.0) {
    publish_absmax_of(a.u, a.n, a.slot_u);
    return;
  }
  const double gamma = a.scal[0], gamma0 = a.scal[7];
  const double rel = sqrt(g) / sqrt(gamma0);
  const bool stop = rel <= tol;
  const double beta = gamma > 0.0 ? g / gamma : 0.0;
  const double th = a.scal[2];
  __syncthreads();  // every thread has read the scalars before workgroup 0 changes them
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    a.scal[9] += 1.0;
    a.scal[10] = rel;
    if (stop) a.scal[8] = 1.0;
    else if (do_update) {
      a.scal[3] = beta;
      a.scal[6] = g;
    }
  }
  if (stop || !do_update) {
    publish_absmax_of(a.u, a.n, a.slot_u);
    return;
  }
  double acc = 0;
  unsigned long long um = 0;
  for (int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x; j < a.n; j += (int64_t)gridDim.x * kThreads) {
    const double uo = a.u[j];
    a.x[j] += th * uo;
    const double un = a.s[j] + beta * uo;
    a.u[j] = un;
    acc += un;
    const unsigned long long b = abs_bits(un);
    um = b > um ? b : um;
  }
  if (a.slot_u) publish_absmax(um, a.slot_u);
  double dummy;
  block_reduce2(acc, 0.0, &a.part[kPartU * kRed + blockIdx.x], &dummy);
}

// x += theta u only (last step, u not needed any more)
__global__ void final_x_kernel(Vecs a, const float* y, float* phi) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= a.n) return;
  const double delta = (double)y[1] - (double)y[0];
  phi[j] = (float)(a.x[j] + a.scal[2] * a.u[j] + delta / (double)a.n);
}

inline unsigned nblocks(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

// ---- hybrid storage of the small members (paired rows, sorted by size) ----
// cnt[r] = size of the small member of pair r; mail[0] = rows with cnt <= thr, mail[1] = 1 if not ascending
__global__ void pair_sizes_kernel(const int32_t* sz, int64_t R, int32_t thr, int32_t* cnt, int64_t* mail) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= R) return;
  const int32_t c = sz[2 * r];
  cnt[r] = c;
  if (c <= thr) atomicAdd((unsigned long long*)&mail[0], 1ull);
  if (r > 0 && sz[2 * (r - 1)] > c) atomicExch((unsigned long long*)&mail[1], 1ull);
}

constexpr int64_t kHybridMinPlayers = 4096;  // below this the plain bit walk is already cheap
constexpr int32_t kDenseDiv = 64;            // pair rows with more than n / 64 players are multiplied as bitmaps

}  // namespace

size_t ds_cgls_arena_bytes(int64_t n, int64_t k) {
  const int64_t KW = (k + 63) / 64;
  // The hybrid storage never exceeds 1.5 x the plain transposed bitmap: the transposed bitmap of the dense pair rows
  // is at most half of it, and the index lists of the sparse rows (needed while their tiles are built) and the tile
  // entries take 4 bytes per set bit of rows with at most n/32 of them each. Plus offsets, the scratch of the two
  // matrix-core products (digit planes, per-group digit sums) and of the tile products (per-group partial vectors,
  // tile counters, the vectors as 64-bit integers).
  const size_t tile_scratch = ds_align((size_t)(2 * (k / 32768) + 160) * n * 8) + ds_align((size_t)32 * k * 8) +
                              ds_align((size_t)(k / 8192 + 160) * (n / 8192 + 2) * 8) + ds_align((size_t)(n + k) * 8);
  const size_t hybrid = 3 * ds_align((size_t)n * KW * 8) + 4 * ds_align((n + 2) * 4) + 2 * ds_align((k + 2) * 4) +
                        ds_align(96 * (size_t)(n > k ? n : k)) + ((size_t)80 << 20) + tile_scratch +
                        4 * ds_scan_arena_bytes(n > k ? n + 1 : k + 1);
  return hybrid + 2 * ds_align(k * 4) + 7 * ds_align(k * 8) + 4 * ds_align(n * 8) + 131072;
}

int ds_solve_cgls_impl(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, const float* y, int paired,
                       double tol, int max_iter, float* phi, int* iters_out, double* relres_out) {
  hipStream_t st = ctx->stream;
  const int64_t W = (n + 63) / 64;
  if (paired && (k & 1)) return ds_fail(ctx, DS_EINVAL, "paired rows need an even row count");
  const int64_t R = paired ? k / 2 : k;
  const int64_t RW = (R + 63) / 64;
  if (tol <= 0) tol = 1e-6;
  if (max_iter <= 0) max_iter = (int)(n < 10000 ? n : 10000);

  int32_t* sz = (int32_t*)ds_arena_alloc(ctx, k * 4);
  float* wc = (float*)ds_arena_alloc(ctx, k * 4);
  double* t = (double*)ds_arena_alloc(ctx, k * 8);
  Vecs a;
  a.n = n; a.k = k; a.R = R; a.paired = paired;
  double* sqw = (double*)ds_arena_alloc(ctx, k * 8);
  a.sqw = sqw;
  a.r = (double*)ds_arena_alloc(ctx, k * 8);
  a.v = (double*)ds_arena_alloc(ctx, k * 8);
  a.d = (double*)ds_arena_alloc(ctx, R * 8);
  a.h = (double*)ds_arena_alloc(ctx, R * 8);
  a.x = (double*)ds_arena_alloc(ctx, n * 8);
  a.u = (double*)ds_arena_alloc(ctx, n * 8);
  a.s = (double*)ds_arena_alloc(ctx, n * 8);
  a.scal = (double*)ds_arena_alloc(ctx, 128);
  a.part = (double*)ds_arena_alloc(ctx, 4 * kRed * 8);
  if (!sz || !wc || !t || !sqw || !a.r || !a.v || !a.d || !a.h || !a.x || !a.u || !a.s || !a.scal || !a.part)
    return ds_fail(ctx, DS_EINTERNAL, "cgls: arena exhausted");

  DS_TRY(ds_row_prep(ctx, Z, k, n, w, y, sz, t, sqw, wc));

  // ---- storage for the two products ----
  // Paired, size-sorted rows of a large game: the small members with at most n/div players become
  // (row, column) entries in 2-D tiles that serve both products through LDS, the denser tail stays a
  // bitmap (rows of Z itself, plus a transposed copy) and is multiplied on the int8 matrix cores; both
  // in fixed point with exact integer sums. Otherwise: plain bitmap and its transpose, set bits walked
  // one by one in fp64.
  bool hybrid = false;
  int64_t Rs = 0, Rd = 0, RdW = 0, nnz_s = 0;
  uint64_t *Zt = nullptr, *Ztd = nullptr;
  ds_mm_plan mm_f = {}, mm_a = {};   // dense rows: forward (Rd x n) and adjoint (n x Rd) products
  ds_tile_plan tiles = {};           // sparse rows: one entry list for both products
  long long *q64u = nullptr, *q64h = nullptr;   // the vectors of the two products as integers (for the sparse rows)
  double *scal_f = nullptr, *scal_a = nullptr;  // [0] scale, [1] maximum slot of the forward / adjoint product
  if (paired && n >= kHybridMinPlayers && n < ((int64_t)1 << 28)) {   // (the matrix-core product addresses rows with 32 bits)
    int32_t* cnt = (int32_t*)ds_arena_alloc(ctx, (R + 1) * 4);
    if (!cnt) return ds_fail(ctx, DS_EINTERNAL, "cgls: arena exhausted");
    DS_HIP(ctx, hipMemsetAsync(ctx->d_mail, 0, 4 * sizeof(int64_t), st));
    const int32_t dense_div = ctx->tuning.cgls_dense_div >= 32 ? ctx->tuning.cgls_dense_div : kDenseDiv;   // below 32 the index lists outgrow the bitmap
    const int32_t thr = (int32_t)(n / dense_div);
    hipLaunchKernelGGL(pair_sizes_kernel, dim3(nblocks(R, 256)), dim3(256), 0, st, sz, R, thr, cnt, ctx->d_mail);
    DS_TRY(ds_mail_fetch(ctx, 4));
    if (ctx->h_mail[1] == 0) {
      hybrid = true;
      Rs = ctx->h_mail[0];
      Rd = R - Rs;
      RdW = (Rd + 63) / 64;
      int32_t* csr_off = (int32_t*)ds_arena_alloc(ctx, (Rs + 2) * 4);
      if (!csr_off) return ds_fail(ctx, DS_EINTERNAL, "cgls: arena exhausted");
      DS_HIP(ctx, hipMemsetAsync(cnt + Rs, 0, 4, st));  // the scan's last slot: total
      DS_TRY(ds_scan_exclusive_i32(ctx, cnt, csr_off, Rs + 1, ctx->d_mail + 2));
      DS_TRY(ds_mail_fetch(ctx, 4));
      nnz_s = ctx->h_mail[2];
      if (nnz_s > 0x7fff0000LL) return ds_fail(ctx, DS_EINTERNAL, "cgls: too many set bits in the sparse rows (%lld)", (long long)nnz_s);
      Ztd = (uint64_t*)ds_arena_alloc(ctx, (size_t)n * (RdW > 0 ? RdW : 1) * 8);
      void* ws_f = ds_arena_alloc(ctx, ds_bit_spmv_mm_ws_bytes(ctx, Rd, n));
      void* ws_a = ds_arena_alloc(ctx, ds_bit_spmv_mm_ws_bytes(ctx, n, Rd));
      void* ws_t = ds_arena_alloc(ctx, ds_tile_ws_bytes(ctx, Rs, n, nnz_s));
      q64u = (long long*)ds_arena_alloc(ctx, n * 8);
      q64h = (long long*)ds_arena_alloc(ctx, (Rs + 1) * 8);
      scal_f = (double*)ds_arena_alloc(ctx, 256);
      int32_t* csr_idx = (int32_t*)ds_arena_alloc(ctx, (nnz_s + 1) * 4);   // (index lists; the tile build keeps the memory)
      if (!Ztd || !ws_f || !ws_a || !ws_t || !q64u || !q64h || !scal_f || !csr_idx) return ds_fail(ctx, DS_EINTERNAL, "cgls: arena exhausted");
      scal_a = scal_f + 16;
      DS_HIP(ctx, hipMemsetAsync(scal_f, 0, 256, st));
      if (Rd > 0) {
        DS_TRY(ds_bit_spmv_mm_prepare(ctx, Rd, n, ws_f, &mm_f));
        DS_TRY(ds_bit_spmv_mm_prepare(ctx, n, Rd, ws_a, &mm_a));
        DS_TRY(ds_bit_transpose(ctx, Z, Rd, n, W, 2 * Rs, 2, Ztd));
      }
      if (Rs > 0) {
        DS_TRY(ds_rows_to_csr(ctx, Z, Rs, n, W, 0, 2, csr_off, csr_idx));
        DS_TRY(ds_tile_build(ctx, Rs, n, nnz_s, thr > 1 ? thr : 1, csr_off, csr_idx, ws_t, &tiles));
      }
      DS_HIP(ctx, hipGetLastError());
    }
  }
  if (!hybrid) {
    Zt = (uint64_t*)ds_arena_alloc(ctx, (size_t)n * RW * 8);
    if (!Zt) return ds_fail(ctx, DS_EINTERNAL, "cgls: arena exhausted");
    DS_TRY(ds_bit_transpose(ctx, Z, R, n, W, 0, paired ? 2 : 1, Zt));
  }
  // Hybrid layout: the vector is brought into fixed point once per product; the sparse rows' tiles and the dense
  // rows' bitmap are multiplied one after the other (side by side on two streams they only competed for memory
  // bandwidth and the iteration took 8 % longer), the dense product adding the sparse result in the adjoint.
  a.slot_u = hybrid ? (unsigned long long*)(scal_f + 1) : nullptr;
  a.slot_h = hybrid ? (unsigned long long*)(scal_a + 1) : nullptr;
  // with_absmax = 0: the kernel that wrote the vector has left its maximum in the product's slot
  // d (sv) == nullptr: the integer partial sums are left for the loop's kernels
  auto forward = [&](const double* u, double* d, int with_absmax) -> int {  // d = (rows) . u
    if (!hybrid) return ds_bit_spmv(ctx, Z, R, n, W, 0, paired ? 2 : 1, u, d);
    DS_TRY(ds_vec_quantize(ctx, u, n, &mm_f, u, u, Rs > 0 ? n : 0, q64u, scal_f, with_absmax));
    if (Rs > 0) DS_TRY(ds_tile_spmv(ctx, &tiles, 0, q64u, scal_f, d, d && Rd == 0 ? 1 : 0));
    if (Rd > 0) DS_TRY(ds_bit_spmv_mm_product(ctx, &mm_f, Z, W, 2 * Rs, 2, scal_f, nullptr, d ? d + Rs : nullptr, d ? 1 : 0));
    return DS_OK;
  };
  auto adjoint = [&](const double* h, double* sv, int with_absmax) -> int {  // s = (rows)^T . h
    if (!hybrid) return ds_bit_spmv(ctx, Zt, n, R, RW, 0, 1, h, sv);
    DS_TRY(ds_vec_quantize(ctx, h, R, &mm_a, h + Rs, h, Rs, q64h, scal_a, with_absmax));
    if (Rs > 0) DS_TRY(ds_tile_spmv(ctx, &tiles, 1, q64h, scal_a, sv, sv && Rd == 0 ? 1 : 0));
    if (Rd > 0) DS_TRY(ds_bit_spmv_mm_product(ctx, &mm_a, Ztd, RdW, 0, 1, scal_a, sv && Rs > 0 ? sv : nullptr, sv, sv ? 1 : 0));
    return DS_OK;
  };
  a.fused = hybrid ? 1 : 0;
  a.Rs = Rs;
  a.fwd = ds_fixed_view_of(&tiles, &mm_f, 0);
  a.adj = ds_fixed_view_of(&tiles, &mm_a, 1);
  a.scal_f = scal_f;
  a.scal_a = scal_a;
  // what one iteration must read of the matrix: the bitmap rows of both orientations and 4 bytes per tile entry, twice
  ctx->cgls_bytes_per_iter = hybrid ? 2.0 * ((double)Rd * (double)W * 8.0 + 4.0 * (double)nnz_s)
                                    : 2.0 * (double)R * (double)W * 8.0;
  DS_HIP(ctx, hipMemsetAsync(a.x, 0, n * 8, st));
  DS_HIP(ctx, hipMemsetAsync(a.u, 0, n * 8, st));
  DS_HIP(ctx, hipMemsetAsync(a.scal, 0, 128, st));

  const unsigned red_n = nblocks(n, kThreads) < (unsigned)kRed ? nblocks(n, kThreads) : (unsigned)kRed;
  const unsigned red_r = nblocks(R, kThreads) < (unsigned)kRed ? nblocks(R, kThreads) : (unsigned)kRed;
  // lanes per entry in the two kernels that add up the products' partial sums: short vectors take 4 or 16, so that
  // enough loads are in flight
  auto lanes_for = [&](int64_t len) { return !hybrid ? 1 : len * 16 <= 262144 ? 16 : len * 4 <= 262144 ? 4 : 1; };
  const int lanes_v = lanes_for(R), lanes_s = lanes_for(n);
  const unsigned grid_v = nblocks(R * lanes_v, kThreads) < (unsigned)kRed ? nblocks(R * lanes_v, kThreads) : (unsigned)kRed;
  const unsigned grid_s = nblocks(n * lanes_s, kThreads) < (unsigned)kRed ? nblocks(n * lanes_s, kThreads) : (unsigned)kRed;
  auto launch_make_v = [&]() {
    if (lanes_v == 16) hipLaunchKernelGGL(loop_make_v_kernel<16>, dim3(grid_v), dim3(kThreads), 0, st, a, (int)red_n);
    else if (lanes_v == 4) hipLaunchKernelGGL(loop_make_v_kernel<4>, dim3(grid_v), dim3(kThreads), 0, st, a, (int)red_n);
    else hipLaunchKernelGGL(loop_make_v_kernel<1>, dim3(grid_v), dim3(kThreads), 0, st, a, (int)red_n);
  };
  auto launch_s_sum = [&]() {
    if (lanes_s == 16) hipLaunchKernelGGL(loop_s_sum_kernel<16>, dim3(grid_s), dim3(kThreads), 0, st, a);
    else if (lanes_s == 4) hipLaunchKernelGGL(loop_s_sum_kernel<4>, dim3(grid_s), dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL(loop_s_sum_kernel<1>, dim3(grid_s), dim3(kThreads), 0, st, a);
  };

  // s_0 = P A^T r_0, u_0 = s_0
  hipLaunchKernelGGL(init_r_kernel, dim3(nblocks(k, 256)), dim3(256), 0, st, a, t);
  hipLaunchKernelGGL(make_h_kernel, dim3(nblocks(R, 256)), dim3(256), 0, st, a);
  DS_TRY(adjoint(a.h, a.s, 1));
  hipLaunchKernelGGL(s_sum_kernel, dim3(red_n), dim3(kThreads), 0, st, a);
  hipLaunchKernelGGL(fin_mean_kernel, dim3(1), dim3(64), 0, st, a, (int)red_n);
  hipLaunchKernelGGL(s_center_kernel, dim3(red_n), dim3(kThreads), 0, st, a);
  hipLaunchKernelGGL(fin_gamma_kernel, dim3(1), dim3(64), 0, st, a, (int)red_n, 1);
  {
    Vecs au = a;  // the partial sums of u live in their own array (the loop's first kernel adds them up)
    au.part = a.part + kPartU * kRed;
    hipLaunchKernelGGL(update_xu_kernel, dim3(red_n), dim3(kThreads), 0, st, au);  // theta = beta = 0: u = s
    hipLaunchKernelGGL(fin_u_kernel, dim3(1), dim3(64), 0, st, au, (int)red_n);
  }
  DS_HIP(ctx, hipGetLastError());
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail, a.scal, 64, hipMemcpyDeviceToHost, st));
  DS_HIP(ctx, hipStreamSynchronize(st));
  const double gamma0 = ((double*)ctx->h_mail)[7];
  int it = 0;
  double rel = gamma0 > 0 ? 1.0 : 0.0;
  bool converged = !(gamma0 > 0);
  DS_TRY(ds_kernel_mark(ctx, 3, 0));
  // The stopping rule runs on the device; the host reads the scalars back every kCheckEvery iterations
  // (kernels queued after the iteration that stopped leave the result alone).
  constexpr int kCheckEvery = 8;
  int launched = 0;
  while (!converged && launched < max_iter) {
    const int burst = max_iter - launched < kCheckEvery ? max_iter - launched : kCheckEvery;
    for (int b = 0; b < burst; ++b) {
      DS_TRY(forward(a.u, hybrid ? nullptr : a.d, launched + b == 0 ? 1 : 0));   // (the first u comes from the set-up, not from the loop's kernel)
      launch_make_v();
      hipLaunchKernelGGL(loop_update_r_kernel, dim3(red_r), dim3(kThreads), 0, st, a, (int)grid_v);
      DS_TRY(adjoint(a.h, hybrid ? nullptr : a.s, 0));
      launch_s_sum();
      hipLaunchKernelGGL(loop_s_center_kernel, dim3(red_n), dim3(kThreads), 0, st, a, (int)grid_s);
      // the last iteration allowed takes no further step: it only evaluates the stopping rule
      hipLaunchKernelGGL(loop_update_xu_kernel, dim3(red_n), dim3(kThreads), 0, st, a, (int)red_n, tol,
                         launched + b + 1 < max_iter ? 1 : 0);
    }
    launched += burst;
    DS_HIP(ctx, hipGetLastError());
    DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail, a.scal, 128, hipMemcpyDeviceToHost, st));
    DS_HIP(ctx, hipStreamSynchronize(st));
    const double* sc = (const double*)ctx->h_mail;
    it = (int)sc[9];
    if (sc[10] > 0.0 || it > 0) rel = sc[10] > 0.0 ? sc[10] : rel;
    if (sc[8] != 0.0) converged = true;
  }
  DS_TRY(ds_kernel_mark(ctx, 3, 1));
  // the last step's x += theta u is folded into the output (theta is 0 if no step was taken)
  hipLaunchKernelGGL(final_x_kernel, dim3(nblocks(n, 256)), dim3(256), 0, st, a, y, phi);
  DS_HIP(ctx, hipGetLastError());
  DS_HIP(ctx, hipStreamSynchronize(st));
  if (iters_out) *iters_out = it;
  if (relres_out) *relres_out = rel;
  if (!converged) {
    ds_fail(ctx, DS_ENOTCONV, "CGLS reached max_iter=%d with relative residual %.3e (tol %.1e)", max_iter, rel, tol);
    return DS_ENOTCONV;
  }
  return DS_OK;
}
