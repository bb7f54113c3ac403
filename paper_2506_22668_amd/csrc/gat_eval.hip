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
template <int NQ>
__device__ __forceinline__ void gat_aggregate_nq(const GatArgs& a, const uint64_t* z, const float* zsrc, int zw,
                                              const float* ssrc, const float* sdst, int H, int F, int rows,
                                              float* dst, const float* bias, bool concat, float* part) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int t = 0; t < rows; ++t) {
    const int e0 = a.row_ptr[t], e1 = a.row_ptr[t + 1];
    const bool coop = e1 - e0 > 2 * 64;
    const int owner = t % kWaves;
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
      for (int base = e0 + (coop ? wave * 64 : 0); base < e1; base += (coop ? kWaves * 64 : 64)) {
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
          int idx[kUnroll];
          bool live[kUnroll];
#pragma unroll
          for (int u = 0; u < kUnroll; ++u) {
            live[u] = mask != 0ull;
            const int i = live[u] ? __ffsll((long long)mask) - 1 : 0;
            if (live[u]) mask &= mask - 1;
            idx[u] = readlane_i(srcn, i);
          }
          float ev[kUnroll][NQ], zv[kUnroll][NQ];
#pragma unroll
          for (int u = 0; u < kUnroll; ++u) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
              ev[u][q] = has[q] ? ssrc[(size_t)idx[u] * H + hd[q]] : 0.f;
              zv[u][q] = has[q] ? zsrc[(size_t)idx[u] * zw + f0 + lane + 64 * q] : 0.f;
            }
          }
#pragma unroll
          for (int u = 0; u < kUnroll; ++u) {
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
            for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, part[(size_t)w * 3 * kColsPerPass + lane + 64 * q]);
            float ls = 0.f, as = 0.f;
            for (int w = 0; w < kWaves; ++w) {  // fixed order: the sum does not depend on timing
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
__device__ __forceinline__ void gat_aggregate(const GatArgs& a, const uint64_t* z, const float* zsrc, int zw,
                                              const float* ssrc, const float* sdst, int H, int F, int rows,
                                              float* dst, const float* bias, bool concat, float* part) {
  if (zw <= 64) gat_aggregate_nq<1>(a, z, zsrc, zw, ssrc, sdst, H, F, rows, dst, bias, concat, part);
  else if (zw <= 128) gat_aggregate_nq<2>(a, z, zsrc, zw, ssrc, sdst, H, F, rows, dst, bias, concat, part);
  else gat_aggregate_nq<4>(a, z, zsrc, zw, ssrc, sdst, H, F, rows, dst, bias, concat, part);
}

__global__ __launch_bounds__(kThreads) void masked_gat_eval_kernel(GatArgs a) {
  extern __shared__ float smem[];
  float* part = smem;  // [kWaves][3][kColsPerPass]
  float* buf = a.buf_lds ? smem + kWaves * 3 * kColsPerPass : a.gws + (size_t)blockIdx.x * a.gws_stride;
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
      for (int i = tid; i < cnt; i += kThreads) bufH[i] = src[i];
      __syncthreads();
    } else {
      const int H = a.heads[0];
      const bool last = L == 1;
      gat_aggregate(a, z, a.P, a.zw[0], a.att1, a.att1 + (size_t)a.V * H, H, a.fh[0], a.rows_out[1],
                    last ? bufT : bufH, a.bias[0], !last, part);
      __syncthreads();
    }
    for (int l = 2; l <= L; ++l) {
      const int rin = a.rows_out[l - 1], din = a.dims[l - 1], zw = a.zw[l - 1], H = a.heads[l - 1], F = a.fh[l - 1];
      const float* Wm = a.Wl[l - 1];
      for (int idx = tid; idx < rin * zw; idx += kThreads) {
        const int r = idx / zw, j = idx - r * zw;
        const float* hr = bufH + (size_t)r * din;
        float s = 0.f;
        for (int i = 0; i < din; ++i) s += hr[i] * Wm[(size_t)i * zw + j];
        bufZ[idx] = s;
      }
      __syncthreads();
      for (int idx = tid; idx < rin * H; idx += kThreads) {
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
      gat_aggregate(a, z, bufZ, zw, bufS, bufS + rin * H, H, F, a.rows_out[l], last ? bufT : bufH, a.bias[l - 1],
                    !last, part);
      __syncthreads();
    }
    // last layer: average the heads of the target's row, add the bias
    {
      const int H = a.heads[L - 1], C = a.fh[L - 1];
      for (int c = tid; c < C; c += kThreads) {
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

struct GatL1Args {
  int32_t V, R1, E1, H, F, zw, zwr, zwp, concat_elu;
  int64_t W, k;
  const int32_t *row_ptr, *col, *eid;
  const float* P;
  const float* att1;
  const float* bias;
  float slope;
  float* Az;      // [(E1 + R1) x zwp]
  int32_t* bad;   // device flag
  const uint64_t* Z;
  float* h1;      // [k][R1][zw]
};

// one workgroup per needed row t
__global__ __launch_bounds__(kThreads) void gat_entry_weights_kernel(GatL1Args g) {
  __shared__ float Mh[64];
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
    if (tid == 0) Mh[h] = mm;
    if (lane == 0 && !(mm - lo <= kAttRange)) atomicOr(g.bad, 1);  // also catches NaN
    __syncthreads();
  }
  for (int ei = e0 + wave; ei <= e1; ei += kWaves) {  // ei == e1: the self term
    const bool self = ei == e1;
    const int src = self ? t : g.col[ei];
    float* out = g.Az + (size_t)(self ? g.E1 + t : ei) * g.zwp;
    for (int c = lane; c < g.zwp; c += 64) {
      float v = 0.f;
      int h = -1;
      if (c < g.zw) h = c / g.F;
      else if (c >= g.zwr && c < g.zwr + g.H) h = c - g.zwr;
      if (h >= 0) {
        const float e = lrelu(ssrc[(size_t)src * g.H + h] + sdst[(size_t)t * g.H + h], g.slope);
        v = __expf(e - Mh[h]);
        if (c < g.zw) v *= g.P[(size_t)src * g.zw + c];
      }
      out[c] = v;
    }
  }
}

// A workgroup takes 64 coalitions (lane = coalition); its waves share the (row, 32-column tile) items.
// v_mfma_f32_32x32x2f32: lane l supplies A[m = l%32][k = l/32] and B[k = l/32][n = l%32]; accumulator
// register i of lane l is D[8*(i/4) + 4*(l/32) + i%4][l%32].
constexpr int kL1Stage = 16;  // entries per step
__global__ __launch_bounds__(kThreads) void masked_gat_layer1_mfma_kernel(GatL1Args g) {
  if (*g.bad != 0) return;
  extern __shared__ float smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  float* den_w = smem + (size_t)wave * (32 * 64 + 2 * 32 * 33);  // [32 heads][64 coalitions]
  float* T_w = den_w + 32 * 64;                                    // two tiles [32 coalitions][33]
  const int FT = g.zwr / 32;
  const int items = g.R1 * FT;
  const int rounds = (items + kWaves - 1) / kWaves;
  const int64_t blocks = (g.k + 63) / 64;
  const size_t h1_stride = (size_t)g.R1 * g.zw;
  for (int64_t blk = blockIdx.x; blk < blocks; blk += gridDim.x) {
    const int64_t row = blk * 64 + lane;
    const uint64_t* zrow = g.Z + (row < g.k ? row : 0) * g.W;  // lanes past the end read row 0 and store nothing
    for (int r = 0; r < rounds; ++r) {
      const int item = r * kWaves + wave;
      const bool live = item < items;
      const int t = live ? item % g.R1 : 0, ft = live ? item / g.R1 : 0;
      float16_t num0, num1, den0, den1;
#pragma unroll
      for (int i = 0; i < 16; ++i) { num0[i] = 0.f; num1[i] = 0.f; den0[i] = 0.f; den1[i] = 0.f; }
      if (live) {
        const int e0 = g.row_ptr[t], e1 = g.row_ptr[t + 1];  // index e1 stands for the self term
        for (int eb = e0; eb <= e1; eb += kL1Stage) {
          const int cnt = e1 + 1 - eb < kL1Stage ? e1 + 1 - eb : kL1Stage;
          int pv = 0;
          if (lane < cnt && eb + lane < e1) pv = g.eid[eb + lane];
          float an[kL1Stage / 2], ad[kL1Stage / 2];
#pragma unroll
          for (int q = 0; q < kL1Stage / 2; ++q) {
            const int ee = eb + 2 * q + half;
            const bool ok = 2 * q + half < cnt;
            const float* ap = g.Az + (size_t)(ee < e1 ? ee : g.E1 + t) * g.zwp;
            an[q] = ok ? ap[ft * 32 + l32] : 0.f;
            ad[q] = ok ? ap[g.zwr + l32] : 0.f;
          }
          float coef[kL1Stage];
#pragma unroll
          for (int i = 0; i < kL1Stage; ++i) {
            coef[i] = 0.f;
            if (i < cnt) {
              const bool self = eb + i == e1;
              const int p = readlane_i(pv, i);
              const bool bit = self || ((zrow[p >> 6] >> (p & 63)) & 1ull);
              coef[i] = bit ? 1.f : 0.f;
            }
          }
#pragma unroll
          for (int q = 0; q < kL1Stage / 2; ++q) {
            if (2 * q < cnt) {
              const float x = coef[2 * q], y = coef[2 * q + 1];
              const float xs = __shfl_xor(x, 32, 64), ys = __shfl_xor(y, 32, 64);
              const float b0 = half ? ys : x;  // coalitions 0..31
              const float b1 = half ? y : xs;  // coalitions 32..63
              num0 = __builtin_amdgcn_mfma_f32_32x32x2f32(an[q], b0, num0, 0, 0, 0);
              num1 = __builtin_amdgcn_mfma_f32_32x32x2f32(an[q], b1, num1, 0, 0, 0);
              den0 = __builtin_amdgcn_mfma_f32_32x32x2f32(ad[q], b0, den0, 0, 0, 0);
              den1 = __builtin_amdgcn_mfma_f32_32x32x2f32(ad[q], b1, den1, 0, 0, 0);
            }
          }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int rr = 8 * (i / 4) + 4 * half + (i % 4);
          den_w[rr * 64 + l32] = den0[i];
          den_w[rr * 64 + 32 + l32] = den1[i];
        }
      }
      __syncthreads();
      if (live) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int fl = 8 * (i / 4) + 4 * half + (i % 4);
          const int f = ft * 32 + fl;
          float v0 = 0.f, v1 = 0.f;
          if (f < g.zw) {
            const int h = f / g.F;
            v0 = num0[i] / den_w[h * 64 + l32];
            v1 = num1[i] / den_w[h * 64 + 32 + l32];
            if (g.concat_elu) {
              const float bb = g.bias ? g.bias[f] : 0.f;
              v0 = elu(v0 + bb);
              v1 = elu(v1 + bb);
            }
          }
          T_w[l32 * 33 + fl] = v0;
          T_w[32 * 33 + l32 * 33 + fl] = v1;
        }
      }
      __syncthreads();
      if (live && ft * 32 + l32 < g.zw) {
#pragma unroll 4
        for (int cc = 0; cc < 32; ++cc) {
          const int c = 2 * cc + half;  // coalition within the block: tile c / 32, column c % 32
          const int64_t rw = blk * 64 + c;
          if (rw < g.k) g.h1[(size_t)rw * h1_stride + (size_t)t * g.zw + ft * 32 + l32] = T_w[(c >> 5) * 32 * 33 + (c & 31) * 33 + l32];
        }
      }
      __syncthreads();
    }
  }
}

constexpr size_t kLdsBufLimit = 64 * 1024;  // buffers beyond this go to global scratch (keeps several workgroups per CU)

struct GatLayout {
  int32_t bufH, bufZ, bufS, bufT;
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

GatLayout gat_layout(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k) {
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
  const size_t fix = (size_t)kWaves * 3 * kColsPerPass * 4;
  g.buf_lds = buf_bytes <= kLdsBufLimit;
  g.lds_bytes = fix + (g.buf_lds ? buf_bytes : 0);
  g.gws_floats = g.buf_lds ? 0 : (int64_t)((buf_bytes / 4 + 63) & ~(size_t)63);
  int occ = (int)((160 * 1024 - 512) / g.lds_bytes);
  if (occ > 2048 / kThreads) occ = 2048 / kThreads;
  if (occ < 1) occ = 1;
  int64_t grid = (int64_t)ctx->num_cus * occ;
  if (grid > k) grid = k;
  if (grid < 1) grid = 1;
  g.grid = (int)grid;
  return g;
}

// the matrix-core path for layer 1 applies to models with at least two layers and enough coalitions
struct GatL1Layout {
  bool use;
  int32_t R1, E1, zwr, zwp;
  size_t az_bytes, h1_bytes, lds_bytes;
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
  q.lds_bytes = (size_t)kWaves * (32 * 64 + 2 * 32 * 33) * 4;
  const int64_t blocks = (k + 63) / 64;
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
  if (g.lds_bytes > 48 * 1024)
    DS_HIP(ctx, hipFuncSetAttribute((const void*)masked_gat_eval_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_bytes));
  hipLaunchKernelGGL(masked_gat_eval_kernel, dim3(grid), dim3(kThreads), g.lds_bytes, ctx->stream, a);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

}  // namespace

size_t ds_gat_eval_arena_bytes(ds_ctx* ctx, const ds_cgraph* cg, int64_t k) {
  const GatLayout g = gat_layout(ctx, cg, k > 1 ? k : 1);
  const size_t W = (cg->info.num_players + 63) / 64;
  const GatL1Layout q = gat_l1_layout(ctx, cg, k);
  return (q.use ? ds_align(q.az_bytes) + ds_align(q.h1_bytes) + 512 : 0) + ds_align((size_t)g.gws_floats * 4 * g.grid) + ds_align((size_t)g.gws_floats * 4) + ds_align(W * 8 + 8) +
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
  const GatLayout g = gat_layout(ctx, cg, k);
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
  const GatL1Layout q = gat_l1_layout(ctx, cg, k);
  GatL1Args l1;
  if (q.use) {
    float* Az = (float*)ds_arena_alloc(ctx, q.az_bytes);
    float* h1 = (float*)ds_arena_alloc(ctx, q.h1_bytes);
    int32_t* bad = (int32_t*)ds_arena_alloc(ctx, 256);
    if (!Az || !h1 || !bad) return ds_fail(ctx, DS_EINTERNAL, "eval: arena exhausted");
    memset(&l1, 0, sizeof(l1));
    l1.V = a.V; l1.R1 = q.R1; l1.E1 = q.E1; l1.H = a.heads[0]; l1.F = a.fh[0]; l1.zw = a.zw[0];
    l1.zwr = q.zwr; l1.zwp = q.zwp; l1.concat_elu = 1;
    l1.W = a.W; l1.k = k;
    l1.row_ptr = a.row_ptr; l1.col = a.col; l1.eid = a.eid;
    l1.P = a.P; l1.att1 = a.att1; l1.bias = a.bias[0]; l1.slope = a.slope;
    l1.Az = Az; l1.bad = bad; l1.Z = Z; l1.h1 = h1;
    a.h1 = h1;
    a.h1_bad = bad;
  }
  DS_TRY(ds_kernel_mark(ctx, 0, 0));
  if (q.use) {
    DS_HIP(ctx, hipMemsetAsync(l1.bad, 0, sizeof(int32_t), ctx->stream));
    hipLaunchKernelGGL(gat_entry_weights_kernel, dim3(q.R1), dim3(kThreads), 0, ctx->stream, l1);
    DS_HIP(ctx, hipGetLastError());
    if (q.lds_bytes > 48 * 1024)
      DS_HIP(ctx, hipFuncSetAttribute((const void*)masked_gat_layer1_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)q.lds_bytes));
    hipLaunchKernelGGL(masked_gat_layer1_mfma_kernel, dim3(q.grid), dim3(kThreads), q.lds_bytes, ctx->stream, l1);
    DS_HIP(ctx, hipGetLastError());
  }
  DS_TRY(gat_launch(ctx, a, g, g.grid));
  return ds_kernel_mark(ctx, 0, 1);
}
