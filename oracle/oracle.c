/*
 * oracle.c - plain C restatement of the oracle for sizes the numpy version cannot finish.
 *
 * TEST INFRASTRUCTURE ONLY (see oracle/__init__.py): it shares no code with the HIP library and is
 * called only by the tests, the smoke check and the benchmark's CPU-baseline leg. Every function is the
 * same definition as its numpy counterpart, written as loops, in fp64; the numpy oracle (which is pinned
 * to the paper's equations and to brute-force Shapley values) is the authority this file is tested
 * against on small inputs (tests/test_oracle_c.py). OpenMP only spreads independent rows over cores.
 *
 *   oc_philox4x32_10   Philox4x32-10 (Salmon et al., SC'11)
 *   oc_plan            size-stratified allocation + weight table (paper: sample-distribution equation)
 *   oc_sample_pairs    complementary pairs of exact-size masks by random keys
 *   oc_gcn_values      f(S): GCN forward on the masked computational graph, all nodes, all layers
 *   oc_cgls            CGLS (paper: Alg. 1 in its standard form) on sqrt(w) Z P from zero
 *   oc_normal_residual |P Z^T W (t - Z psi)| / |P Z^T W t| for a given phi (property check at any size)
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ENUM_MAX_PLAYERS 24

/* ------------------------------------------------------------------ Philox */
void oc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
  for (int r = 0; r < 10; ++r) {
    if (r > 0) {
      k0 += 0x9E3779B9u;
      k1 += 0xBB67AE85u;
    }
    uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------ plan */
static double rho(int64_t n, int64_t s) { return (double)(n - 1) / ((double)s * (double)(n - s)); }

/* b[0..H], wtab[0..H] (H = n/2); returns k (rows), *enumerate set. */
int64_t oc_plan(int64_t n, int64_t n_samples, int64_t* b, float* wtab, int32_t* enumerate) {
  const int64_t H = n / 2;
  const int en = (n <= ENUM_MAX_PLAYERS && n_samples >= ((int64_t)1 << n));
  *enumerate = en;
  for (int64_t s = 0; s <= H; ++s) { b[s] = 0; wtab[s] = 0.0f; }
  if (en) {
    double binom = 1.0;
    for (int64_t s = 1; s <= H; ++s) {
      binom = binom * (double)(n - s + 1) / (double)s;
      wtab[s] = (float)(rho(n, s) / binom);
    }
    return (int64_t)1 << n;
  }
  const int64_t k = 2 * (n_samples / 2), K = k / 2 - 1;
  double* c = (double*)calloc((size_t)H + 1, sizeof(double));
  double acc = 0.0;
  for (int64_t s = 1; s <= H; ++s) {
    double r = rho(n, s);
    acc = acc + ((2 * s == n) ? r : 2.0 * r);
    c[s] = acc;
  }
  for (int64_t s = 1; s < H; ++s) b[s] = (int64_t)floor((double)K * (c[s] / acc) + 0.5);
  if (H >= 1) b[H] = K;
  for (int64_t s = 1; s <= H; ++s) {
    int64_t m = (b[s] - b[s - 1]) * ((2 * s == n) ? 2 : 1);
    if (m > 0) wtab[s] = (float)(rho(n, s) / (double)m);
  }
  free(c);
  return k;
}

/* ------------------------------------------------------------------ masks */
static int cmp_u64(const void* a, const void* b) {
  uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}

/* Rows 2*(r - pair_begin), +1 for pairs pair_begin <= r < pair_end. Z: uint64[rows][W], W = ceil(n/64). */
int oc_sample_pairs(int64_t n, int64_t n_samples, uint64_t seed, uint32_t tag, int64_t pair_begin, int64_t pair_end,
                    uint64_t* Z, float* w, int32_t* sz) {
  const int64_t H = n / 2, W = (n + 63) / 64;
  int64_t* b = (int64_t*)malloc(((size_t)H + 1) * sizeof(int64_t));
  float* wtab = (float*)malloc(((size_t)H + 1) * sizeof(float));
  int32_t en;
  oc_plan(n, n_samples, b, wtab, &en);
  const uint64_t tail = (n & 63) ? ((1ull << (n & 63)) - 1ull) : ~0ull;
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
#pragma omp parallel
  {
    uint64_t* comp = (uint64_t*)malloc((size_t)(n + 4) * sizeof(uint64_t));
#pragma omp for schedule(dynamic, 8)
    for (int64_t r = pair_begin; r < pair_end; ++r) {
      uint64_t* small = Z + 2 * (r - pair_begin) * W;
      uint64_t* big = small + W;
      const int64_t o = 2 * (r - pair_begin);
      memset(small, 0, (size_t)W * 8);
      int64_t s;
      float wt;
      if (en) {
        small[0] = (uint64_t)r;
        s = __builtin_popcountll((uint64_t)r);
        int64_t cls = s < n - s ? s : n - s;
        wt = cls == 0 ? 0.0f : wtab[cls];
      } else if (r == 0) {
        s = 0;
        wt = 0.0f;
      } else {
        s = 1;
        while (b[s] < r) ++s; /* small size of pair r: min{s : b_s >= r} */
        wt = wtab[s];
        for (int64_t q = 0; 4 * q < n; ++q) {
          uint32_t ctr[4] = {(uint32_t)q, (uint32_t)r, (uint32_t)((uint64_t)r >> 32), tag}, out[4];
          oc_philox4x32_10(ctr, key, out);
          for (int i = 0; i < 4 && 4 * q + i < n; ++i) comp[4 * q + i] = ((uint64_t)out[i] << 32) | (uint64_t)(4 * q + i);
        }
        qsort(comp, (size_t)n, sizeof(uint64_t), cmp_u64); /* ascending (key, column) */
        for (int64_t i = 0; i < s; ++i) {
          const uint64_t j = comp[i] & 0xFFFFFFFFull;
          small[j >> 6] |= 1ull << (j & 63);
        }
      }
      for (int64_t wd = 0; wd < W; ++wd) big[wd] = ~small[wd] & (wd == W - 1 ? tail : ~0ull);
      w[o] = wt;
      w[o + 1] = wt;
      sz[o] = (int32_t)s;
      sz[o + 1] = (int32_t)(n - s);
    }
    free(comp);
  }
  free(b);
  free(wtab);
  return 0;
}

/* ------------------------------------------------------------------ GCN value function */
static double round_bf16(double x) {
  float f = (float)x;
  uint32_t u;
  memcpy(&u, &f, 4);
  u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}

/*
 * y[i] = f(S_i) for `rows` coalitions. Computational graph: V nodes (target = node 0), n players with
 * local end points (psrc, pdst); undirected players switch both directions. X: double[V][dims[0]].
 * Wcat: the L weight matrices one after another (row-major d_{l-1} x d_l); bias_cat: NULL or the L bias
 * vectors one after another. score: 0 softmax probability, 1 logit, of class pred_class.
 * Every layer is evaluated on every node: A~ = A_S + I, A^ = D^-1/2 A~ D^-1/2, H <- act(A^ H W + b).
 * bf16 != 0 (a diagnostic mode, not what parity is judged against): in layers 2..L both operands of the dense
 * transform (A^ H and W_l) are rounded to bfloat16 and the products summed exactly; layer 1 is not rounded.
 */
int oc_gcn_values(int32_t V, int64_t n, const int32_t* psrc, const int32_t* pdst, int32_t directed, const double* X,
                  int32_t L, const int32_t* dims, const double* Wcat, const double* bias_cat, int32_t bf16, int32_t score,
                  int32_t pred_class, const uint64_t* Z, int64_t rows, double* y, double* logits_out /* rows x d_L or NULL */) {
  const int64_t W64 = (n + 63) / 64;
  int dmax = 0;
  for (int l = 0; l <= L; ++l)
    if (dims[l] > dmax) dmax = dims[l];
#pragma omp parallel
  {
    double* H = (double*)malloc((size_t)V * dmax * sizeof(double));
    double* A = (double*)malloc((size_t)V * dmax * sizeof(double));
    double* T = (double*)malloc((size_t)V * dmax * sizeof(double));
    double* dinv = (double*)malloc((size_t)V * sizeof(double));
    double* Wr = (double*)malloc((size_t)dmax * dmax * sizeof(double));
#pragma omp for schedule(dynamic, 1)
    for (int64_t i = 0; i < rows; ++i) {
      const uint64_t* z = Z + i * W64;
      for (int v = 0; v < V; ++v) dinv[v] = 1.0; /* self-loop */
      for (int64_t p = 0; p < n; ++p)
        if ((z[p >> 6] >> (p & 63)) & 1ull) {
          dinv[pdst[p]] += 1.0;
          if (!directed) dinv[psrc[p]] += 1.0;
        }
      for (int v = 0; v < V; ++v) dinv[v] = 1.0 / sqrt(dinv[v]);
      memcpy(H, X, (size_t)V * dims[0] * sizeof(double));
      const double* Wl = Wcat;
      const double* bl = bias_cat;
      for (int l = 1; l <= L; ++l) {
        const int din = dims[l - 1], dout = dims[l];
        const int round_ops = bf16 && l >= 2; /* the first product is shared by all coalitions and stays unrounded */
        const double* Wuse = Wl;
        if (round_ops) {
          for (int q = 0; q < din * dout; ++q) Wr[q] = round_bf16(Wl[q]);
          Wuse = Wr;
        }
        /* A = A^ H */
        for (int v = 0; v < V; ++v)
          for (int q = 0; q < din; ++q) A[(size_t)v * din + q] = dinv[v] * dinv[v] * H[(size_t)v * din + q];
        for (int64_t p = 0; p < n; ++p)
          if ((z[p >> 6] >> (p & 63)) & 1ull) {
            const int s = psrc[p], d = pdst[p];
            const double c = dinv[s] * dinv[d];
            for (int q = 0; q < din; ++q) A[(size_t)d * din + q] += c * H[(size_t)s * din + q];
            if (!directed)
              for (int q = 0; q < din; ++q) A[(size_t)s * din + q] += c * H[(size_t)d * din + q];
          }
        /* T = A W (operands rounded to bfloat16 in the reduced-precision layers), then H = T */
        for (int v = 0; v < V; ++v)
          for (int j = 0; j < dout; ++j) {
            double s = 0.0;
            for (int q = 0; q < din; ++q) {
              const double a = round_ops ? round_bf16(A[(size_t)v * din + q]) : A[(size_t)v * din + q];
              s += a * Wuse[(size_t)q * dout + j];
            }
            T[(size_t)v * dout + j] = s;
          }
        memcpy(H, T, (size_t)V * dout * sizeof(double));
        for (int v = 0; v < V; ++v)
          for (int j = 0; j < dout; ++j) {
            double s = H[(size_t)v * dout + j] + (bl ? bl[j] : 0.0);
            H[(size_t)v * dout + j] = (l < L && s < 0.0) ? 0.0 : s;
          }
        Wl += (size_t)din * dout;
        if (bl) bl += dout;
      }
      const int C = dims[L];
      const double* lg = H; /* node 0 = target */
      if (logits_out) memcpy(logits_out + i * C, lg, (size_t)C * sizeof(double));
      if (score == 1) {
        y[i] = lg[pred_class];
      } else {
        double m = lg[0], sum = 0.0;
        for (int c = 1; c < C; ++c)
          if (lg[c] > m) m = lg[c];
        for (int c = 0; c < C; ++c) sum += exp(lg[c] - m);
        y[i] = exp(lg[pred_class] - m) / sum;
      }
    }
    free(H); free(A); free(T); free(dinv); free(Wr);
  }
  return 0;
}

/* threads the parallel loops of this file use (reported beside timings of the oracle) */
int oc_threads(void) { return omp_get_max_threads(); }

/* ------------------------------------------------------------------ least squares */
static void row_targets(int64_t n, int64_t k, const uint64_t* Z, const float* w, const double* y, double* t, double* sq) {
  const int64_t W64 = (n + 63) / 64;
  const double f0 = y[0], delta = y[1] - y[0];
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < k; ++i) {
    int64_t c = 0;
    for (int64_t wd = 0; wd < W64; ++wd) c += __builtin_popcountll(Z[i * W64 + wd]);
    t[i] = i < 2 ? 0.0 : y[i] - f0 - (delta / (double)n) * (double)c;
    sq[i] = i < 2 ? 0.0 : sqrt((double)w[i]);
  }
}

/* v = sq .* (Z u) */
static void fwd(int64_t n, int64_t k, const uint64_t* Z, const double* sq, const double* u, double* v) {
  const int64_t W64 = (n + 63) / 64;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t i = 0; i < k; ++i) {
    double s = 0.0;
    for (int64_t wd = 0; wd < W64; ++wd) {
      uint64_t word = Z[i * W64 + wd];
      while (word) {
        s += u[wd * 64 + __builtin_ctzll(word)];
        word &= word - 1;
      }
    }
    v[i] = sq[i] * s;
  }
}

/* s = P Z^T (sq .* r). Rows are split statically over the threads and the per-thread sums are added in
 * thread order, so the result does not change from run to run on one machine. */
static void adj(int64_t n, int64_t k, const uint64_t* Z, const double* sq, const double* r, double* s) {
  const int64_t W64 = (n + 63) / 64;
  int nthreads = 1;
#pragma omp parallel
  {
#pragma omp single
    nthreads = omp_get_num_threads();
  }
  double* loc = (double*)calloc((size_t)nthreads * (size_t)n, sizeof(double));
#pragma omp parallel num_threads(nthreads)
  {
    double* mine = loc + (size_t)omp_get_thread_num() * (size_t)n;
#pragma omp for schedule(static)
    for (int64_t i = 0; i < k; ++i) {
      const double g = sq[i] * r[i];
      if (g == 0.0) continue;
      for (int64_t wd = 0; wd < W64; ++wd) {
        uint64_t word = Z[i * W64 + wd];
        while (word) {
          mine[wd * 64 + __builtin_ctzll(word)] += g;
          word &= word - 1;
        }
      }
    }
  }
  for (int64_t j = 0; j < n; ++j) {
    double acc = 0.0;
    for (int t = 0; t < nthreads; ++t) acc += loc[(size_t)t * (size_t)n + j];
    s[j] = acc;
  }
  free(loc);
  double mean = 0.0;
  for (int64_t j = 0; j < n; ++j) mean += s[j];
  mean /= (double)n;
  for (int64_t j = 0; j < n; ++j) s[j] -= mean;
}

static double dot(int64_t m, const double* a, const double* b) {
  double s = 0.0;
  for (int64_t i = 0; i < m; ++i) s += a[i] * b[i];
  return s;
}

int oc_cgls(int64_t n, int64_t k, const uint64_t* Z, const float* w, const double* y, double tol, int64_t max_iter,
            double* phi, int64_t* iters, double* relres) {
  double *t = malloc(k * 8), *sq = malloc(k * 8), *r = malloc(k * 8), *v = malloc(k * 8);
  double *x = calloc(n, 8), *s = malloc(n * 8), *u = malloc(n * 8);
  row_targets(n, k, Z, w, y, t, sq);
  for (int64_t i = 0; i < k; ++i) r[i] = sq[i] * t[i];
  adj(n, k, Z, sq, r, s);
  memcpy(u, s, n * 8);
  double gamma0 = dot(n, s, s), gamma = gamma0, rel = gamma0 > 0 ? 1.0 : 0.0;
  int64_t it = 0;
  while (gamma0 > 0 && it < max_iter) {
    fwd(n, k, Z, sq, u, v);
    const double dl = dot(k, v, v);
    if (dl == 0.0) break;
    const double th = gamma / dl;
    for (int64_t j = 0; j < n; ++j) x[j] += th * u[j];
    for (int64_t i = 0; i < k; ++i) r[i] -= th * v[i];
    adj(n, k, Z, sq, r, s);
    const double gn = dot(n, s, s);
    ++it;
    rel = sqrt(gn) / sqrt(gamma0);
    if (rel <= tol) break;
    const double beta = gn / gamma;
    for (int64_t j = 0; j < n; ++j) u[j] = s[j] + beta * u[j];
    gamma = gn;
  }
  const double delta = y[1] - y[0];
  for (int64_t j = 0; j < n; ++j) phi[j] = x[j] + delta / (double)n;
  *iters = it;
  *relres = rel;
  free(t); free(sq); free(r); free(v); free(x); free(s); free(u);
  return 0;
}

/* |P Z^T W (t - Z psi)| / |P Z^T W t| with psi = phi - delta/n: what CGLS drives below tol. */
double oc_normal_residual(int64_t n, int64_t k, const uint64_t* Z, const float* w, const double* y, const double* phi) {
  double *t = malloc(k * 8), *sq = malloc(k * 8), *r = malloc(k * 8), *v = malloc(k * 8);
  double *psi = malloc(n * 8), *s = malloc(n * 8);
  row_targets(n, k, Z, w, y, t, sq);
  const double delta = y[1] - y[0];
  for (int64_t j = 0; j < n; ++j) psi[j] = phi[j] - delta / (double)n;
  for (int64_t i = 0; i < k; ++i) r[i] = sq[i] * t[i];
  adj(n, k, Z, sq, r, s);
  const double g0 = dot(n, s, s);
  fwd(n, k, Z, sq, psi, v);
  for (int64_t i = 0; i < k; ++i) r[i] -= v[i];
  adj(n, k, Z, sq, r, s);
  const double g1 = dot(n, s, s);
  free(t); free(sq); free(r); free(v); free(psi); free(s);
  return g0 > 0 ? sqrt(g1) / sqrt(g0) : 0.0;
}
