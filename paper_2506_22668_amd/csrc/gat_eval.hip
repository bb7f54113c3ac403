// Masked GAT inference of the target node for many edge coalitions.
//
// Paper, "GNN Models" / GAT scaling experiment: the second model family is a graph
// attention network (layer of Velickovic et al., cited by the paper). Under a
// coalition S, with Z = H^(l-1) W_l and z_i^h the slice of head h,
//   e_ij^h = LeakyReLU(a_dst^h . z_i^h + a_src^h . z_j^h),  j in N_S(i) + {i}
//   out_i^h = sum_j softmax_j(e_ij^h) z_j^h
// hidden layers concatenate heads (+bias, ELU), the last layer averages them (+bias).
//
// One workgroup evaluates one coalition at a time. As for the GCN, layer l is only
// produced on the nodes within L-l hops of the target (a prefix of the local node
// order), and the first transform Z_1 = X_c W_1 together with its attention scalars
// is coalition-independent and computed once per target. The soft-max of a row is
// accumulated in one pass with a running maximum, so a row's entries are read once;
// a wave walks the set bits of 64 entries at a time, lanes hold feature columns.
#include <algorithm>

#include "internal.h"
#include "solve_common.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kUnroll = 8;         // active entries gathered per step
constexpr int kColsPerPass = 256;  // feature columns a wave covers per pass over a row (4 per lane)

struct GatArgs {
  int32_t V, n, L, score;
  const int32_t* pred_ptr;
  int32_t dims[DS_MAX_LAYERS + 1];      // output width of every layer
  int32_t zw[DS_MAX_LAYERS], heads[DS_MAX_LAYERS], fh[DS_MAX_LAYERS];
  int32_t rows_out[DS_MAX_LAYERS + 1];  // rows produced by layer l (1..L): nodes within L-l hops
  int64_t W, k;
  const int32_t *row_ptr, *col, *eid;
  const float* P;     // [V x zw_1]
  const float* att1;  // neighbour scalars [V x heads_1], then receiver scalars [V x heads_1]
  const float* Wl[DS_MAX_LAYERS];
  const float* bias[DS_MAX_LAYERS];
  const float* asrc[DS_MAX_LAYERS];
  const float* adst[DS_MAX_LAYERS];
  float slope;
  const uint64_t* Z;
  float* y;
  float* logits_out;
  float* gws;          // per-workgroup global scratch when the buffers do not fit LDS
  int64_t gws_stride;  // floats per workgroup
  int32_t bufH, bufZ, bufS, bufT;  // floats
  int32_t buf_lds;
  const float* h1;      // optional: layer-1 output of every coalition [k][rows_out[1]][dims[1]] (matrix-core path)
  const int32_t* h1_bad; // device flag: non-zero means h1 was not produced (attention range too wide)
};

__device__ __forceinline__ int readlane_i(int v, int l) { return __builtin_amdgcn_readlane(v, l); }

__device__ __forceinline__ float lrelu(float x, float slope) { return x > 0.f ? x : slope * x; }
__device__ __forceinline__ float elu(float x) { return x > 0.f ? x : expm1f(x); }

// Attention aggregation of rows [0, rows) for one layer.
//   zsrc [.. x zw]: transformed rows; ssrc/sdst [.. x H]: attention scalars of the neighbour / receiver role.
//   concat: dst[t, f] = ELU(out + bias[f]) over all zw columns; otherwise dst[t, h*F + c] = raw head outputs
//   (the caller averages them).
// Short rows go to one wave each; a long row is shared by all waves, whose partial (max, sum, acc)
// triples meet in LDS and are merged by the owner in a fixed order.
template <int NQ, int WAVES>
__device__ __forceinline__ void gat_aggregate_nq(const GatArgs& a, const uint64_t* z, const float* zsrc, int zw,
                                              const float* ssrc, const float* sdst, int H, int F, int rows,
                                              float* dst, const float* bias, bool concat, float* part) {
  constexpr int UNROLL = WAVES == 1 ? 4 : kUnroll;  // the one-wave variant trades gather depth for occupancy
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int t = 0; t < rows; ++t) {
    const int e0 = a.row_ptr[t], e1 = a.row_ptr[t + 1];
    const bool coop = e1 - e0 > 2 * 64;
    const int owner = t % WAVES;
    if (!coop && owner != wave) continue;
    for (int f0 = 0; f0 < zw; f0 += 64 * NQ) {
      bool has[NQ];
      int hd[NQ];
      float sd[NQ], m[NQ], l[NQ], acc[NQ];
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        const int f = f0 + lane + 64 * q;
        has[q] = f < zw;
        hd[q] = has[q] ? f / F : 0;
        sd[q] = has[q] ? sdst[(size_t)t * H + hd[q]] : 0.f;
        if (wave == owner) {  // the self term starts the running soft-max
          m[q] = has[q] ? lrelu(ssrc[(size_t)t * H + hd[q]] + sd[q], a.slope) : 0.f;
          l[q] = 1.f;
          acc[q] = has[q] ? zsrc[(size_t)t * zw + f] : 0.f;
        } else {
          m[q] = -INFINITY;
          l[q] = 0.f;
          acc[q] = 0.f;
        }
      }
      for (int base = e0 + (coop ? wave * 64 : 0); base < e1; base += (coop ? WAVES * 64 : 64)) {
        const int e = base + lane;
        int srcn = 0;
        bool bit = false;
        if (e < e1) {
          const int p = a.eid[e];
          srcn = a.col[e];
          bit = (z[p >> 6] >> (p & 63)) & 1ull;
        }
        unsigned long long mask = __ballot(bit);
        // eight active entries per step: their loads are independent and issue back to back
        while (mask) {
          int idx[UNROLL];
          bool live[UNROLL];
#pragma unroll
          for (int u = 0; u < UNROLL; ++u) {
            live[u] = mask != 0ull;
            const int i = live[u] ? __ffsll((long long)mask) - 1 : 0;
            if (live[u]) mask &= mask - 1;
            idx[u] = readlane_i(srcn, i);
          }
          float ev[UNROLL][NQ], zv[UNROLL][NQ];
#pragma unroll
          for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
              ev[u][q] = has[q] ? ssrc[(size_t)idx[u] * H + hd[q]] : 0.f;
              zv[u][q] = has[q] ? zsrc[(size_t)idx[u] * zw + f0 + lane + 64 * q] : 0.f;
            }
          }
#pragma unroll
          for (int u = 0; u < UNROLL; ++u) {
            if (!live[u]) break;  // uniform across the wave
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
              // running soft-max: of the two factors exp(m - max) and exp(e - max) one is always 1
              const float ee = lrelu(ev[u][q] + sd[q], a.slope);
              const float d = ee - m[q];
              const float x = __expf(-fabsf(d));
              const float sc = d > 0.f ? x : 1.f, pe = d > 0.f ? 1.f : x;
              l[q] = l[q] * sc + pe;
              acc[q] = acc[q] * sc + pe * zv[u][q];
              m[q] = fmaxf(m[q], ee);
            }
          }
        }
      }
      if (coop) {
        float* mine = part + (size_t)wave * 3 * kColsPerPass + lane;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
          mine[64 * q] = m[q];
          mine[kColsPerPass + 64 * q] = l[q];
          mine[2 * kColsPerPass + 64 * q] = acc[q];
        }
        __syncthreads();
        if (wave == owner) {
#pragma unroll
          for (int q = 0; q < NQ; ++q) {
            float mm = -INFINITY;
            for (int w = 0; w < WAVES; ++w) mm = fmaxf(mm, part[(size_t)w * 3 * kColsPerPass + lane + 64 * q]);
            float ls = 0.f, as = 0.f;
            for (int w = 0; w < WAVES; ++w) {  // fixed order: the sum does not depend on timing
              const float* o = part + (size_t)w * 3 * kColsPerPass + lane + 64 * q;
              const float sc = __expf(o[0] - mm);  // exp(-inf) = 0 for a wave that saw nothing
              ls += o[kColsPerPass] * sc;
              as += o[2 * kColsPerPass] * sc;
            }
            l[q] = ls;
            acc[q] = as;
          }
        }
      }
      if (wave == owner) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
          if (!has[q]) continue;
          const int f = f0 + lane + 64 * q;
          float v = acc[q] / l[q];
          if (concat) {
            if (bias) v += bias[f];
            v = elu(v);
          }
          dst[(size_t)t * zw + f] = v;
        }
      }
      if (coop) __syncthreads();
    }
  }
}

// the number of 64-column groups a lane carries is fixed at compile time (1, 2 or 4)
template <int WAVES>
__device__ __forceinline__ void gat_aggregate(const GatArgs& a, const uint64_t* z, const float* zsrc, int zw,
                                              const float* ssrc, const float* sdst, int H, int F, int rows,
                                              float* dst, const float* bias, bool concat, float* part) {
  if (zw <= 64) gat_aggregate_nq<1, WAVES>(a, z, zsrc, zw, ssrc, sdst, H, F, rows, dst, bias, concat, part);
  else if (zw <= 128 || WAVES == 1)  // the one-wave variant walks wide rows in passes of 128 columns: fewer registers
    gat_aggregate_nq<2, WAVES>(a, z, zsrc, zw, ssrc, sdst, H, F, rows, dst, bias, concat, part);
  else gat_aggregate_nq<4, WAVES>(a, z, zsrc, zw, ssrc, sdst, H, F, rows, dst, bias, concat, part);
}

// THREADS = 256: a workgroup per coalition (every layer here); THREADS = 64: a wave per coalition, used when
// layer 1 comes precomputed and only the small later layers are left.
template <int THREADS>
__device__ __forceinline__ void masked_gat_eval_body(const GatArgs& a) {
  constexpr int WAVES = THREADS / 64;
  extern __shared__ float smem[];
  float* part = smem;  // [WAVES][3][kColsPerPass]
  float* buf = a.buf_lds ? smem + WAVES * 3 * kColsPerPass : a.gws + (size_t)blockIdx.x * a.gws_stride;
  float* bufH = buf;
  float* bufZ = bufH + a.bufH;
  float* bufS = bufZ + a.bufZ;
  float* bufT = bufS + a.bufS;
  const int tid = threadIdx.x;
  const int L = a.L;

  for (int64_t row = blockIdx.x; row < a.k; row += gridDim.x) {
    const uint64_t* z = a.Z + row * a.W;
    // layer 1: already produced for all coalitions on the matrix cores, or aggregated here
    if (a.h1 && *a.h1_bad == 0) {
      const int cnt = a.rows_out[1] * a.dims[1];
      const float* src = a.h1 + (size_t)row * cnt;
      for (int i = tid; i < cnt; i += THREADS) bufH[i] = src[i];
      __syncthreads();
    } else {
      const int H = a.heads[0];
      const bool last = L == 1;
      gat_aggregate<WAVES>(a, z, a.P, a.zw[0], a.att1, a.att1 + (size_t)a.V * H, H, a.fh[0], a.rows_out[1],
                    last ? bufT : bufH, a.bias[0], !last, part);
      __syncthreads();
    }
    for (int l = 2; l <= L; ++l) {
      const int rin = a.rows_out[l - 1], din = a.dims[l - 1], zw = a.zw[l - 1], H = a.heads[l - 1], F = a.fh[l - 1];
      const float* Wm = a.Wl[l - 1];
      for (int idx = tid; idx < rin * zw; idx += THREADS) {
        const int r = idx / zw, j = idx - r * zw;
        const float* hr = bufH + (size_t)r * din;
        float s = 0.f;
        for (int i = 0; i < din; ++i) s += hr[i] * Wm[(size_t)i * zw + j];
        bufZ[idx] = s;
      }
      __syncthreads();
      for (int idx = tid; idx < rin * H; idx += THREADS) {
        const int r = idx / H, h = idx - r * H;
        const float* zr = bufZ + (size_t)r * zw + h * F;
        const float *as = a.asrc[l - 1] + h * F, *ad = a.adst[l - 1] + h * F;
        float s0 = 0.f, s1 = 0.f;
        for (int i = 0; i < F; ++i) {
          s0 += as[i] * zr[i];
          s1 += ad[i] * zr[i];
        }
        bufS[idx] = s0;
        bufS[rin * H + idx] = s1;
      }
      __syncthreads();
      const bool last = l == L;
      gat_aggregate<WAVES>(a, z, bufZ, zw, bufS, bufS + rin * H, H, F, a.rows_out[l], last ? bufT : bufH, a.bias[l - 1],
                    !last, part);
      __syncthreads();
    }
    // last layer: average the heads of the target's row, add the bias
    {
      const int H = a.heads[L - 1], C = a.fh[L - 1];
      for (int c = tid; c < C; c += THREADS) {
        float s = 0.f;
        for (int h = 0; h < H; ++h) s += bufT[h * C + c];
        s = s / (float)H;
        if (a.bias[L - 1]) s += a.bias[L - 1][c];
        bufH[c] = s;
      }
      __syncthreads();
    }
    if (tid < 64) {
      const int C = a.dims[L];
      float m = -INFINITY;
      for (int c = tid; c < C; c += 64) m = fmaxf(m, bufH[c]);
      for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
      float s = 0.f;
      for (int c = tid; c < C; c += 64) s += expf(bufH[c] - m);
      for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      if (tid == 0) {
        const float zc = bufH[*a.pred_ptr];
        a.y[row] = a.score == DS_SCORE_LOGIT ? zc : expf(zc - m) / s;
      }
      if (a.logits_out)
        for (int c = tid; c < C; c += 64) a.logits_out[row * C + c] = bufH[c];
    }
    __syncthreads();
  }
}

template <int THREADS>
__global__ __launch_bounds__(THREADS) void masked_gat_eval_kernel(GatArgs a) {
  masked_gat_eval_body<THREADS>(a);
}

// the wave-per-coalition variant lives on latency hiding: ask for at least six waves per SIMD
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(6, 8))) void masked_gat_eval_wave_kernel(GatArgs a) {
  masked_gat_eval_body<64>(a);
}

// s_src[v, h] = a_src^h . z_v^h and s_dst[v, h] = a_dst^h . z_v^h for the shared first transform
__global__ void gat_att_scalars_kernel(const float* P, const float* asrc, const float* adst, int V, int H, int F,
                                       float* out) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= V * H) return;
  const int v = idx / H, h = idx - v * H;
  const float* zr = P + (size_t)v * H * F + h * F;
  float s0 = 0.f, s1 = 0.f;
  for (int i = 0; i < F; ++i) {
    s0 += asrc[h * F + i] * zr[i];
    s1 += adst[h * F + i] * zr[i];
  }
  out[idx] = s0;
  out[(size_t)V * H + idx] = s1;
}


// ---------------- layer 1 of all coalitions at once on the matrix cores ----------------
//
// The attention logits of layer 1, e_tj^h, do not depend on the coalition: only the set of
// neighbours the soft-max runs over does. With M_t^h the maximum of e_tj^h over the whole row (self
// included) and p_tj^h = exp(e_tj^h - M_t^h),
//   out_t^h[f] = ( sum_{j active} p_tj^h z_j^h[f] ) / ( sum_{j active} p_tj^h ),
// so numerator and denominator of row t are products of a coalition-independent matrix
// (columns x entries) with the 0/1 matrix (entries x coalitions): dense contractions.
//   Az[e][0 .. zw)        = p_e^{h(f)} * z_{src e}[f]       (entry e of a needed row; the self term of row t
//   Az[e][zwr .. zwr + H) = p_e^h                             is stored as row E1 + t)
// zwr = zw rounded up to 32; the row stride is zwr + 32. The self term is always active, so the
// denominator is at least p_tt > 0; if some p would fall below exp(-70) the flag is raised and the
// per-coalition kernel computes layer 1 itself with a running maximum.
typedef float float16_t __attribute__((ext_vector_type(16)));
constexpr float kAttRange = 70.f;
__device__ __forceinline__ bool ft_in_range(int ft, int l32, int zw) { return ft * 32 + l32 < zw; }

struct GatL1Args {
  int32_t V, R1, E1, H, F, zw, zwr, zwp, concat_elu;
  int64_t W, k;
  const int32_t *row_ptr, *col, *eid;
  const float* P;
  const float* att1;
  const float* bias;
  float slope;
  float* Az;      // [(E1 + R1) x zwp]
  float* rowmax;  // [R1 x H]
  int32_t* bad;   // device flag
  const uint64_t* Zt;  // optional: transposed masks [n][KW], word blk of row p = bit p of coalitions 64 blk ..
  int64_t KW;
  float* h1;      // [k][R1][zw]
};

// row maxima M[t][h] over the whole row (self included); one workgroup per needed row t
__global__ __launch_bounds__(kThreads) void gat_row_max_kernel(GatL1Args g) {
  __shared__ float red[kWaves];
  const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int e0 = g.row_ptr[t], e1 = g.row_ptr[t + 1];
  const float* ssrc = g.att1;
  const float* sdst = g.att1 + (size_t)g.V * g.H;
  for (int h = 0; h < g.H; ++h) {
    const float sd = sdst[(size_t)t * g.H + h];
    float m = lrelu(ssrc[(size_t)t * g.H + h] + sd, g.slope);
    float lo = m;
    for (int e = e0 + tid; e < e1; e += kThreads) {
      const float v = lrelu(ssrc[(size_t)g.col[e] * g.H + h] + sd, g.slope);
      m = fmaxf(m, v);
      lo = fminf(lo, v);
    }
    for (int o = 32; o > 0; o >>= 1) {
      m = fmaxf(m, __shfl_xor(m, o, 64));
      lo = fminf(lo, __shfl_xor(lo, o, 64));
    }
    if (lane == 0) red[wave] = m;
    __syncthreads();
    float mm = red[0];
    for (int w = 1; w < kWaves; ++w) mm = fmaxf(mm, red[w]);
    if (tid == 0) g.rowmax[t * g.H + h] = mm;
    if (lane == 0 && !(mm - lo <= kAttRange)) atomicOr(g.bad, 1);  // also catches NaN
    __syncthreads();
  }
}

// one wave per entry of the needed rows (the self terms come after the E1 entries)
__global__ __launch_bounds__(kThreads) void gat_entry_weights_kernel(GatL1Args g) {
  const int lane = threadIdx.x & 63;
  const int ei = blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (ei >= g.E1 + g.R1) return;
  int t, src;
  if (ei >= g.E1) {
    t = ei - g.E1;
    src = t;
  } else {
    int lo = 0, hi = g.R1 - 1;  // last row whose first entry is <= ei
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (g.row_ptr[mid] <= ei) lo = mid; else hi = mid - 1;
    }
    t = lo;
    src = g.col[ei];
  }
  const float* ssrc = g.att1;
  const float* sdst = g.att1 + (size_t)g.V * g.H;
  float* out = g.Az + (size_t)ei * g.zwp;
  for (int c = lane; c < g.zwp; c += 64) {
    float v = 0.f;
    int h = -1;
    if (c < g.zw) h = c / g.F;
    else if (c >= g.zwr && c < g.zwr + g.H) h = c - g.zwr;
    if (h >= 0) {
      const float e = lrelu(ssrc[(size_t)src * g.H + h] + sdst[(size_t)t * g.H + h], g.slope);
      v = __expf(e - g.rowmax[t * g.H + h]);
      if (c < g.zw) v *= g.P[(size_t)src * g.zw + c];
    }
    out[c] = v;
  }
}

// A workgroup takes 128 coalitions, 32 per wave, and every wave walks all needed rows for its own
// coalitions, so the waves carry identical work whatever the row lengths are (a hub row is no imbalance).
// v_mfma_f32_32x32x2f32: lane l supplies A[m = l%32][k = l/32] and B[k = l/32][n = l%32]; accumulator
// register i of lane l is D[8*(i/4) + 4*(l/32) + i%4][l%32]. Per row a wave accumulates up to three
// 32-column tiles of the numerator plus the denominator tile (one row per head).
// The 0/1 operand comes from the transposed mask matrix: a word of player p holds the bits of 64
// coalitions, so the words of the needed entries (staged in LDS once per block of coalitions) serve every
// lane and no cross-lane traffic is needed: lane l takes bit (32 (wave%2) + l%32) of the word of entry
// 2q + l/32. The A operand of the next step is loaded while the current step multiplies.
constexpr int kL1Stage = 16;        // entries per step
constexpr int kL1Tiles = 3;         // numerator tiles per pass
constexpr int kL1MaxEntries = 4096; // entries of the needed rows whose mask words fit the LDS stage
constexpr int kL1WaveFloats = 32 * 33 + 32 * 33;
__global__ __launch_bounds__(kThreads) void masked_gat_layer1_mfma_kernel(GatL1Args g) {
  if (*g.bad != 0) return;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_l1[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int wsel_word = wave >> 1, wsel_shift = 32 * (wave & 1) + l32;
  uint64_t* bitsL = (uint64_t*)smem_l1;  // [2][E1 + 2]: mask words of the needed entries, then all-ones, then zero
  const int bstride = g.E1 + 2;
  float* den_w = (float*)(smem_l1 + (((size_t)2 * bstride * 8 + 15) & ~(size_t)15)) + (size_t)wave * kL1WaveFloats;
  float* T_w = den_w + 32 * 33;  // one tile [32 coalitions][33]
  const uint64_t* my_bits = bitsL + (size_t)wsel_word * bstride;
  const int FT = g.zwr / 32;
  const int64_t blocks = (g.k + 127) / 128;
  const size_t h1_stride = (size_t)g.R1 * g.zw;
  for (int64_t blk = blockIdx.x; blk < blocks; blk += gridDim.x) {
    __syncthreads();
    for (int i = tid; i < 2 * g.E1; i += kThreads) {
      const int wd = i >= g.E1 ? 1 : 0, e = i - wd * g.E1;
      const int64_t kw = 2 * blk + wd;
      bitsL[(size_t)wd * bstride + e] = kw < g.KW ? g.Zt[(size_t)g.eid[e] * g.KW + kw] : 0ull;
    }
    if (tid < 2) {
      bitsL[(size_t)tid * bstride + g.E1] = ~0ull;    // the self term is always active
      bitsL[(size_t)tid * bstride + g.E1 + 1] = 0ull; // past the end of a row
    }
    __syncthreads();
    const int64_t row_base = blk * 128 + wave * 32;
    for (int t = 0; t < g.R1; ++t) {
      const int e0 = g.row_ptr[t], e1 = g.row_ptr[t + 1];  // index e1 stands for the self term
      const size_t self_row = (size_t)(g.E1 + t) * g.zwp;
      for (int fg = 0; fg < FT; fg += kL1Tiles) {
        const int nt = FT - fg < kL1Tiles ? FT - fg : kL1Tiles;
        float16_t num[kL1Tiles], den;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          den[i] = 0.f;
#pragma unroll
          for (int j = 0; j < kL1Tiles; ++j) num[j][i] = 0.f;
        }
        const float* az = g.Az + l32;
        float an[kL1Stage / 2][kL1Tiles], ad[kL1Stage / 2];
#pragma unroll
        for (int q = 0; q < kL1Stage / 2; ++q) {  // rows past the end are clamped to the self row and masked by B = 0
          const int ee = e0 + 2 * q + half;
          const float* ap = az + (ee < e1 ? (size_t)ee * g.zwp : self_row);
#pragma unroll
          for (int j = 0; j < kL1Tiles; ++j) an[q][j] = ap[(fg + (j < nt ? j : 0)) * 32];
          ad[q] = ap[g.zwr];
        }
        for (int eb = e0; eb <= e1; eb += kL1Stage) {
          float an2[kL1Stage / 2][kL1Tiles], ad2[kL1Stage / 2];
#pragma unroll
          for (int q = 0; q < kL1Stage / 2; ++q) {
            const int ee = eb + kL1Stage + 2 * q + half;
            const float* ap = az + (ee < e1 ? (size_t)ee * g.zwp : self_row);
#pragma unroll
            for (int j = 0; j < kL1Tiles; ++j) an2[q][j] = ap[(fg + (j < nt ? j : 0)) * 32];
            ad2[q] = ap[g.zwr];
          }
#pragma unroll
          for (int q = 0; q < kL1Stage / 2; ++q) {
            const int ee = eb + 2 * q + half;
            const uint64_t wsel = my_bits[ee < e1 ? ee : (ee == e1 ? g.E1 : g.E1 + 1)];
            const float bq = (float)((uint32_t)(wsel >> wsel_shift) & 1u);
            den = __builtin_amdgcn_mfma_f32_32x32x2f32(ad[q], bq, den, 0, 0, 0);
            num[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(an[q][0], bq, num[0], 0, 0, 0);
            if (nt > 1) num[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(an[q][1], bq, num[1], 0, 0, 0);
            if (nt > 2) num[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(an[q][2], bq, num[2], 0, 0, 0);
          }
#pragma unroll
          for (int q = 0; q < kL1Stage / 2; ++q) {
            ad[q] = ad2[q];
#pragma unroll
            for (int j = 0; j < kL1Tiles; ++j) an[q][j] = an2[q][j];
          }
        }
        // denominators to LDS as [head][coalition], so that every column finds its head's
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 16; ++i) den_w[(8 * (i / 4) + 4 * half + (i % 4)) * 33 + l32] = den[i];
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kL1Tiles; ++j) {
          if (j < nt) {
            const int ft = fg + j;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int fl = 8 * (i / 4) + 4 * half + (i % 4);
              const int f = ft * 32 + fl;
              float v = 0.f;
              if (f < g.zw) {
                v = num[j][i] * __frcp_rn(den_w[(f / g.F) * 33 + l32]);
                if (g.concat_elu) {
                  v += g.bias ? g.bias[f] : 0.f;
                  v = v > 0.f ? v : __expf(v) - 1.f;
                }
              }
              T_w[l32 * 33 + fl] = v;
            }
          }
          __syncthreads();
          if (j < nt && ft_in_range(fg + j, l32, g.zw)) {
#pragma unroll 4
            for (int cc = 0; cc < 16; ++cc) {
              const int c = 2 * cc + half;  // coalition of this wave
              const int64_t rw = row_base + c;
              if (rw < g.k) g.h1[(size_t)rw * h1_stride + (size_t)t * g.zw + (fg + j) * 32 + l32] = T_w[c * 33 + l32];
            }
          }
          __syncthreads();
        }
      }
    }
  }
}

constexpr size_t kLdsBufLimit = 64 * 1024;  // buffers beyond this go to global scratch (keeps several workgroups per CU)

struct GatLayout {
  int32_t bufH, bufZ, bufS, bufT;
  int threads;
  bool buf_lds;
  size_t lds_bytes;
  int64_t gws_floats;
  int grid;
};

void gat_rows(const ds_ctx* ctx, const ds_cgraph* cg, int32_t rows_out[DS_MAX_LAYERS + 1]) {
  const int L = ctx->L, hops = cg->info.hops;
  rows_out[0] = (int32_t)cg->info.num_nodes;
  for (int l = 1; l <= L; ++l) {
    int h = L - l;
    if (h > hops) h = hops;
    rows_out[l] = (int32_t)cg->info.ball[h];
  }
}

GatLayout gat_layout(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k, int threads = kThreads) {
  int32_t rows_out[DS_MAX_LAYERS + 1];
  gat_rows(ctx, cg, rows_out);
  const int L = ctx->L;
  int64_t Hm = ctx->dims[L], Zm = 1, Sm = 1;
  for (int l = 1; l < L; ++l) Hm = std::max<int64_t>(Hm, (int64_t)rows_out[l] * ctx->dims[l]);
  for (int l = 2; l <= L; ++l) {
    Zm = std::max<int64_t>(Zm, (int64_t)rows_out[l - 1] * ctx->gat.zw[l - 1]);
    Sm = std::max<int64_t>(Sm, 2 * (int64_t)rows_out[l - 1] * ctx->gat.heads[l - 1]);
  }
  GatLayout g;
  g.bufH = (int32_t)Hm;
  g.bufZ = (int32_t)Zm;
  g.bufS = (int32_t)Sm;
  g.bufT = (int32_t)((int64_t)rows_out[L] * ctx->gat.zw[L - 1]);
  const size_t buf_bytes = ((size_t)Hm + Zm + Sm + g.bufT) * 4;
  const size_t fix = (size_t)(threads / 64) * 3 * kColsPerPass * 4;
  g.threads = threads;
  g.buf_lds = buf_bytes <= kLdsBufLimit;
  g.lds_bytes = fix + (g.buf_lds ? buf_bytes : 0);
  g.gws_floats = g.buf_lds ? 0 : (int64_t)((buf_bytes / 4 + 63) & ~(size_t)63);
  int occ = (int)((160 * 1024 - 512) / g.lds_bytes);
  if (occ > 2048 / threads) occ = 2048 / threads;
  if (occ < 1) occ = 1;
  int64_t grid = (int64_t)ctx->num_cus * occ;
  if (grid > k) grid = k;
  if (grid < 1) grid = 1;
  g.grid = (int)grid;
  return g;
}

// the matrix-core path for layer 1 applies to models with at least two layers and enough coalitions
struct GatL1Layout {
  bool use, transpose;
  int32_t R1, E1, zwr, zwp;
  int64_t KW;
  size_t az_bytes, h1_bytes, zt_bytes, lds_bytes;
  int grid;
};

GatL1Layout gat_l1_layout(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k) {
  GatL1Layout q;
  memset(&q, 0, sizeof(q));
  const int L = ctx->L, hops = cg->info.hops;
  if (L < 2 || k < 256 || cg->info.num_players < 1 || ctx->gat.heads[0] > 32) return q;
  const int h = L - 1 < hops ? L - 1 : hops;
  q.R1 = (int32_t)cg->info.ball[h];
  const int64_t E1 = cg->ball_entries[h];
  if (E1 < 0 || E1 > 0x7fffff00LL) return q;
  q.E1 = (int32_t)E1;
  q.zwr = (ctx->gat.zw[0] + 31) & ~31;
  q.zwp = q.zwr + 32;
  q.az_bytes = ((size_t)E1 + q.R1) * q.zwp * 4;
  q.h1_bytes = (size_t)k * q.R1 * ctx->gat.zw[0] * 4;
  if (q.az_bytes > ((size_t)256 << 20) || q.h1_bytes > ((size_t)2 << 30)) return q;
  // the 0/1 operand is read from a transposed copy of the mask matrix (one word = one player for 64
  // coalitions); when that copy would be out of proportion the per-coalition kernel does every layer
  const size_t W = (size_t)(cg->info.num_players + 63) / 64;
  q.KW = (k + 63) / 64;
  q.transpose = true;
  if ((size_t)k * W * 8 > ((size_t)1 << 30) || q.E1 > kL1MaxEntries) return q;
  q.zt_bytes = (size_t)cg->info.num_players * q.KW * 8;
  q.lds_bytes = (((size_t)2 * (q.E1 + 2) * 8 + 15) & ~(size_t)15) + (size_t)kWaves * kL1WaveFloats * 4;
  const int64_t blocks = (k + 127) / 128;
  const int64_t cap = (int64_t)ctx->num_cus * 2;
  q.grid = (int)(blocks < cap ? blocks : cap);
  q.use = true;
  return q;
}

void gat_fill(const ds_ctx* ctx, const ds_cgraph* cg, const GatLayout& g, GatArgs* a) {
  memset(a, 0, sizeof(*a));
  a->V = (int32_t)cg->info.num_nodes;
  a->n = (int32_t)cg->info.num_players;
  a->L = ctx->L;
  for (int l = 0; l <= ctx->L; ++l) a->dims[l] = ctx->dims[l];
  gat_rows(ctx, cg, a->rows_out);
  for (int l = 0; l < ctx->L; ++l) {
    a->zw[l] = ctx->gat.zw[l];
    a->heads[l] = ctx->gat.heads[l];
    a->fh[l] = ctx->gat.fh[l];
    a->Wl[l] = ctx->W[l];
    a->bias[l] = ctx->bias[l];
    a->asrc[l] = ctx->gat.att_src[l];
    a->adst[l] = ctx->gat.att_dst[l];
  }
  a->slope = ctx->gat.slope;
  a->W = (cg->info.num_players + 63) / 64;
  a->row_ptr = cg->row_ptr;
  a->col = cg->col;
  a->eid = cg->eid;
  a->P = cg->P;
  a->att1 = cg->att;
  a->bufH = g.bufH;
  a->bufZ = g.bufZ;
  a->bufS = g.bufS;
  a->bufT = g.bufT;
  a->buf_lds = g.buf_lds ? 1 : 0;
  a->gws_stride = g.gws_floats;
}

int gat_launch(ds_ctx* ctx, const GatArgs& a, const GatLayout& g, int grid) {
  if (g.threads == 64) {
    if (g.lds_bytes > 48 * 1024)
      DS_HIP(ctx, hipFuncSetAttribute((const void*)masked_gat_eval_wave_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_bytes));
    hipLaunchKernelGGL(masked_gat_eval_wave_kernel, dim3(grid), dim3(64), g.lds_bytes, ctx->stream, a);
  } else {
    if (g.lds_bytes > 48 * 1024)
      DS_HIP(ctx, hipFuncSetAttribute((const void*)masked_gat_eval_kernel<kThreads>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_bytes));
    hipLaunchKernelGGL(masked_gat_eval_kernel<kThreads>, dim3(grid), dim3(kThreads), g.lds_bytes, ctx->stream, a);
  }
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

}  // namespace

size_t ds_gat_eval_arena_bytes(ds_ctx* ctx, const ds_cgraph* cg, int64_t k) {
  const GatL1Layout q = gat_l1_layout(ctx, cg, k);
  const GatLayout g = gat_layout(ctx, cg, k > 1 ? k : 1, q.use ? 64 : kThreads);
  const GatLayout g1 = gat_layout(ctx, cg, 1);
  const size_t W = (cg->info.num_players + 63) / 64;
  return (q.use ? ds_align(q.az_bytes) + ds_align(q.h1_bytes) + ds_align(q.zt_bytes + 8) + ds_align((size_t)q.R1 * 32 * 4) + 1024 : 0) +
         ds_align((size_t)g1.gws_floats * 4) + ds_align((size_t)g.gws_floats * 4 * g.grid) + ds_align((size_t)g.gws_floats * 4) + ds_align(W * 8 + 8) +
         ds_align(ctx->dims[ctx->L] * 4 + 8) + 1024;
}

int ds_gat_prepare_model(ds_ctx* ctx, ds_cgraph* cg) {
  if (cg->d0 != ctx->dims[0]) return ds_fail(ctx, DS_EINVAL, "feature width %d does not match the model's input width %d", cg->d0, ctx->dims[0]);
  if (cg->model_version == ctx->model_version) return DS_OK;
  const int H = ctx->gat.heads[0], F = ctx->gat.fh[0];
  if (cg->d1 != ctx->gat.zw[0] || cg->att_heads != H)
    return ds_fail(ctx, DS_EINVAL, "the computational graph was extracted for another model (first transform width %d, now %d): extract again", cg->d1, ctx->gat.zw[0]);
  const int V = (int)cg->info.num_nodes;
  DS_TRY(ds_launch_first_transform(ctx, cg->Xc, ctx->W[0], cg->P, V, ctx->dims[0], ctx->gat.zw[0], 0));
  hipLaunchKernelGGL(gat_att_scalars_kernel, dim3((V * H + 255) / 256), dim3(256), 0, ctx->stream, cg->P,
                     ctx->gat.att_src[0], ctx->gat.att_dst[0], V, H, F, cg->att);
  DS_HIP(ctx, hipGetLastError());
  // predicted class: evaluate the full coalition once and take the first maximum
  const int64_t n = cg->info.num_players;
  const int64_t W = (n + 63) / 64;
  const int C = ctx->dims[ctx->L];
  const GatLayout g = gat_layout(ctx, cg, 1);
  uint64_t* zfull = (uint64_t*)ds_arena_alloc(ctx, W * 8 + 8);
  float* logits = (float*)ds_arena_alloc(ctx, C * 4 + 8);
  float* gws = g.gws_floats ? (float*)ds_arena_alloc(ctx, (size_t)g.gws_floats * 4) : nullptr;
  if (!zfull || !logits || (g.gws_floats && !gws)) return ds_fail(ctx, DS_EINTERNAL, "prepare: arena exhausted");
  DS_TRY(ds_launch_full_mask(ctx, zfull, W, n));
  GatArgs a;
  gat_fill(ctx, cg, g, &a);
  a.Z = zfull;
  a.k = 1;
  a.y = logits + C;
  a.logits_out = logits;
  a.gws = gws;
  a.score = DS_SCORE_LOGIT;
  DS_HIP(ctx, hipMemsetAsync(cg->d_pred, 0, sizeof(int32_t), ctx->stream));
  a.pred_ptr = cg->d_pred;
  DS_TRY(gat_launch(ctx, a, g, 1));
  DS_TRY(ds_launch_argmax(ctx, logits, C, cg->d_pred));
  cg->pred_class = -1;
  cg->model_version = ctx->model_version;
  return DS_OK;
}

int ds_gat_eval_impl(ds_ctx* ctx, ds_cgraph* cg, const uint64_t* Z, int64_t k, int score, float* y) {
  DS_TRY(ds_gat_prepare_model(ctx, cg));
  if (k <= 0) return DS_OK;
  const GatL1Layout q = gat_l1_layout(ctx, cg, k);
  const GatLayout g = gat_layout(ctx, cg, k, q.use ? 64 : kThreads);
  float* gws = nullptr;
  if (g.gws_floats) {
    gws = (float*)ds_arena_alloc(ctx, (size_t)g.gws_floats * 4 * g.grid);
    if (!gws) return ds_fail(ctx, DS_EINTERNAL, "eval: arena exhausted");
  }
  GatArgs a;
  gat_fill(ctx, cg, g, &a);
  a.Z = Z;
  a.k = k;
  a.y = y;
  a.logits_out = nullptr;
  a.gws = gws;
  a.score = score;
  a.pred_ptr = cg->d_pred;
  GatL1Args l1;
  uint64_t* Zt_w = nullptr;
  if (q.use) {
    float* Az = (float*)ds_arena_alloc(ctx, q.az_bytes);
    float* h1 = (float*)ds_arena_alloc(ctx, q.h1_bytes);
    int32_t* bad = (int32_t*)ds_arena_alloc(ctx, 256);
    float* rowmax = (float*)ds_arena_alloc(ctx, (size_t)q.R1 * 32 * 4);
    uint64_t* Zt = q.transpose ? (uint64_t*)ds_arena_alloc(ctx, q.zt_bytes + 8) : nullptr;
    if (!Az || !h1 || !bad || !rowmax || (q.transpose && !Zt)) return ds_fail(ctx, DS_EINTERNAL, "eval: arena exhausted");
    memset(&l1, 0, sizeof(l1));
    l1.V = a.V; l1.R1 = q.R1; l1.E1 = q.E1; l1.H = a.heads[0]; l1.F = a.fh[0]; l1.zw = a.zw[0];
    l1.zwr = q.zwr; l1.zwp = q.zwp; l1.concat_elu = 1;
    l1.W = a.W; l1.k = k;
    l1.row_ptr = a.row_ptr; l1.col = a.col; l1.eid = a.eid;
    l1.P = a.P; l1.att1 = a.att1; l1.bias = a.bias[0]; l1.slope = a.slope;
    l1.Az = Az; l1.bad = bad; l1.h1 = h1;
    l1.rowmax = rowmax; l1.Zt = Zt; l1.KW = q.KW;
    Zt_w = Zt;
    a.h1 = h1;
    a.h1_bad = bad;
  }
  DS_TRY(ds_kernel_mark(ctx, 0, 0));
  if (q.use) {
    DS_HIP(ctx, hipMemsetAsync(l1.bad, 0, sizeof(int32_t), ctx->stream));
    hipLaunchKernelGGL(gat_row_max_kernel, dim3(q.R1), dim3(kThreads), 0, ctx->stream, l1);
    hipLaunchKernelGGL(gat_entry_weights_kernel, dim3((q.E1 + q.R1 + kWaves - 1) / kWaves), dim3(kThreads), 0, ctx->stream, l1);
    DS_HIP(ctx, hipGetLastError());
    if (q.transpose) DS_TRY(ds_bit_transpose(ctx, Z, k, cg->info.num_players, a.W, 0, 1, Zt_w));
    if (q.lds_bytes > 48 * 1024)
      DS_HIP(ctx, hipFuncSetAttribute((const void*)masked_gat_layer1_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)q.lds_bytes));
    hipLaunchKernelGGL(masked_gat_layer1_mfma_kernel, dim3(q.grid), dim3(kThreads), q.lds_bytes, ctx->stream, l1);
    DS_HIP(ctx, hipGetLastError());
  }
  DS_TRY(gat_launch(ctx, a, g, g.grid));
  return ds_kernel_mark(ctx, 0, 1);
}
