// Masked GCN inference of the target node for many edge coalitions.
//
// Paper, "Distributed Model Prediction": the GNN is evaluated once per sampled
// sub-graph; the paper batches by stacking block-diagonal copies of the adjacency
// and multiplying element-wise with a block-diagonal mask. Here the mask bits are
// read in place by one of three kernels, chosen by the size of the problem:
//   * few coalitions, or graphs too wide for the others: one workgroup per coalition, every per-coalition
//     intermediate in LDS (masked_gcn_eval_kernel);
//   * short mask rows (up to 12,288 players): one coalition per lane, 64 per workgroup, masks, degrees and the
//     local CSR on chip, the first layer on the matrix cores; per-coalition activations of later layers go
//     through a per-workgroup scratch in global memory (masked_gcn_eval_batched_kernel);
//   * long mask rows: a streaming kernel reads each row once (of a complementary pair: only one member) and
//     reduces it to node degrees and the bits of the entries layer 1 reads (stream_degrees_kernel); the
//     one-coalition-per-lane kernel then runs the layers from those compact arrays.
//
// GCN layer under a coalition S (Kipf & Welling, as cited by the paper; degrees
// renormalised per coalition):  A~ = A_S + I, d_i = row sum of A~,
//   H^l = act( D^-1/2 A~ D^-1/2 H^(l-1) W_l + b_l ).
// The result is identical to evaluating all of G_c, but only the rows that can
// reach the target are produced: layer l is computed on the nodes within L-l hops.
// Layer 1 uses the coalition-independent product P = X_c W_1 (computed once per
// target with MFMA) and aggregates it; layers >= 2 aggregate, then transform.
#include "internal.h"
#include <type_traits>

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef short short4_t __attribute__((ext_vector_type(4)));

struct EvalArgs {
  int32_t V, n, L, directed, score, bf16;
  const int32_t* pred_ptr;  // device: index of the class whose score is returned
  int32_t dims[DS_MAX_LAYERS + 1];
  int32_t rows_out[DS_MAX_LAYERS + 1];  // rows produced by layer l (1..L)
  int64_t W, k;
  const int32_t *row_ptr, *col, *eid;
  const int2* pl;  // player end points (local ids)
  const float* P;
  const float* Wl[DS_MAX_LAYERS];
  const float* bias[DS_MAX_LAYERS];
  const uint64_t* Z;
  float* y;
  float* logits_out;  // optional: [k x d_L]
  float* gws;         // per-workgroup global scratch when LDS is too small
  int64_t gws_stride; // floats per workgroup
  int32_t bufA_floats, bufB_floats;
};

__device__ __forceinline__ float bf16_round(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest even (finite inputs)
  return __uint_as_float(u & 0xFFFF0000u);
}

__device__ __forceinline__ short bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (short)(u >> 16);
}

__device__ __forceinline__ int block_sum_int(int v, int* sh) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) t += sh[i];
  __syncthreads();
  return t;
}

__device__ __forceinline__ int readlane_i(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ __forceinline__ float readlane_f(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

// dst[t, :] = rs[t] * ( sum_{active e in row t} rs[col e] * src[col e, :] + rs[t] * src[t, :] ) (+bias, ReLU)
// One wave per row; lanes hold features; the 64 entries of a chunk test their mask
// bits together and the set bits of the ballot are walked in order.
__device__ __forceinline__ void aggregate_rows(const EvalArgs& a, const uint64_t* z, const float* rs,
                                               const float* src, int stride, int rows, int width,
                                               float* dst, const float* bias, bool relu, float* part) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int t = 0; t < rows; ++t) {
    const int e0 = a.row_ptr[t], e1 = a.row_ptr[t + 1];
    // a long row (a hub) is shared by all waves of the workgroup, 64 entries at a time each, and its
    // partial sums meet in LDS; short rows go to one wave each
    const bool coop = e1 - e0 > 2 * 64;
    const int owner = t % kWaves;
    if (!coop && owner != wave) continue;
    const float rst = rs[t];
    for (int f0 = 0; f0 < width; f0 += 256) {
      const int f = f0 + lane;
      float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
      const bool h0 = f < width, h1 = f + 64 < width, h2 = f + 128 < width, h3 = f + 192 < width;
      for (int base = e0 + (coop ? wave * 64 : 0); base < e1; base += (coop ? kWaves * 64 : 64)) {
        const int e = base + lane;
        int srcn = 0;
        float coef = 0.f;
        bool bit = false;
        if (e < e1) {
          const int p = a.eid[e];
          srcn = a.col[e];
          bit = (z[p >> 6] >> (p & 63)) & 1ull;
          coef = rs[srcn];
        }
        unsigned long long mask = __ballot(bit);
        // eight active entries per step: their row loads are independent and issue back to back
        while (mask) {
          int idx[8];
          float cf[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const bool live = mask != 0ull;
            const int i = live ? __ffsll((long long)mask) - 1 : 0;
            if (live) mask &= mask - 1;
            idx[u] = readlane_i(srcn, i);
            cf[u] = live ? readlane_f(coef, i) : 0.f;
          }
          float v0[8], v1[8], v2[8], v3[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const float* sp = src + (size_t)idx[u] * stride + f;
            v0[u] = h0 ? sp[0] : 0.f;
            v1[u] = h1 ? sp[64] : 0.f;
            v2[u] = h2 ? sp[128] : 0.f;
            v3[u] = h3 ? sp[192] : 0.f;
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            acc0 += cf[u] * v0[u];
            acc1 += cf[u] * v1[u];
            acc2 += cf[u] * v2[u];
            acc3 += cf[u] * v3[u];
          }
        }
      }
      if (coop) {
        float* mine = part + wave * 256 + lane;
        mine[0] = acc0;
        mine[64] = acc1;
        mine[128] = acc2;
        mine[192] = acc3;
        __syncthreads();
        if (wave == owner) {
          acc0 = acc1 = acc2 = acc3 = 0.f;
#pragma unroll
          for (int w = 0; w < kWaves; ++w) {  // fixed order: the sum does not depend on timing
            const float* o = part + w * 256 + lane;
            acc0 += o[0];
            acc1 += o[64];
            acc2 += o[128];
            acc3 += o[192];
          }
        }
      }
      if (wave == owner) {
        const float* sp = src + (size_t)t * stride + f;
        float* dp = dst + (size_t)t * width + f;
        float v;
        if (h0) { v = rst * (acc0 + rst * sp[0]);   if (bias) v += bias[f];       dp[0]   = relu ? fmaxf(v, 0.f) : v; }
        if (h1) { v = rst * (acc1 + rst * sp[64]);  if (bias) v += bias[f + 64];  dp[64]  = relu ? fmaxf(v, 0.f) : v; }
        if (h2) { v = rst * (acc2 + rst * sp[128]); if (bias) v += bias[f + 128]; dp[128] = relu ? fmaxf(v, 0.f) : v; }
        if (h3) { v = rst * (acc3 + rst * sp[192]); if (bias) v += bias[f + 192]; dp[192] = relu ? fmaxf(v, 0.f) : v; }
      }
      if (coop) __syncthreads();
    }
  }
}

// dst[t, j] = act( sum_i q[t, i] * W[i, j] + b[j] ), the per-coalition dense transform of a layer ("Distributed Model
// Prediction": the |V_c| d^2 term), on the matrix cores: a wave takes a 32-row x 32-column tile of the result,
// v_mfma_f32_32x32x2f32 with lane l supplying q[row l%32][i l/32] and W[i l/32][column l%32]; in the bf16 configuration
// both operands are rounded to bfloat16 (nearest even) and v_mfma_f32_32x32x8bf16_1k accumulates in fp32.
__device__ __forceinline__ void transform_rows(const float* q, int rows, int din, int dout, const float* Wm,
                                               const float* bias, bool relu, bool bf16, float* dst) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r = lane & 31, half = lane >> 5;
  const int tn = (dout + 31) / 32, tm = (rows + 31) / 32;
  for (int tile = wave; tile < tm * tn; tile += kWaves) {
    const int m0 = (tile / tn) * 32, n0 = (tile - (tile / tn) * tn) * 32;
    const int am = m0 + r, bn = n0 + r;
    const bool aok = am < rows, bok = bn < dout;
    const float* qr = q + (size_t)(aok ? am : 0) * din;
    const float* wc = Wm + (bok ? bn : 0);
    float16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    for (int k0 = 0; k0 < din; k0 += 8) {
      float x[4], w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int kk = k0 + (bf16 ? 4 * half + u : 2 * u + half);
        const bool ok = kk < din;
        x[u] = (ok && aok) ? qr[kk] : 0.f;
        w[u] = (ok && bok) ? wc[(size_t)kk * dout] : 0.f;
      }
      if (bf16) {
        short4_t av, bv;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          av[u] = bf16_bits(x[u]);
          bv[u] = bf16_bits(w[u]);
        }
        acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(av, bv, acc, 0, 0, 0);
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[u], w[u], acc, 0, 0, 0);
      }
    }
    // accumulator register i of lane l is the result's [row 8*(i/4) + 4*(l/32) + i%4][column l%32]
    if (bok) {
      const float bj = bias ? bias[bn] : 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int t = m0 + 8 * (i / 4) + 4 * half + (i % 4);
        if (t < rows) {
          const float v = acc[i] + bj;
          dst[(size_t)t * dout + bn] = relu ? fmaxf(v, 0.f) : v;
        }
      }
    }
  }
}

template <bool RS_LDS, bool BUF_LDS>
__global__ __launch_bounds__(kThreads) void masked_gcn_eval_kernel(EvalArgs a) {
  extern __shared__ float smem[];
  int* red = (int*)smem;  // 16 ints of reduction scratch, then the per-wave partial sums of shared rows
  float* part = smem + 16;
  float* rs;
  float* bufA;
  float* bufB;
  {
    float* lds = smem + 16 + kWaves * 256;
    float* g = a.gws + (size_t)blockIdx.x * a.gws_stride;
    if (RS_LDS) { rs = lds; lds += a.V; } else { rs = g; g += a.V; }
    if (BUF_LDS) { bufA = lds; bufB = lds + a.bufA_floats; } else { bufA = g; bufB = g + a.bufA_floats; }
  }
  const int tid = threadIdx.x;
  const int64_t W = a.W;
  const uint64_t tail_mask = (a.n & 63) ? ((1ull << (a.n & 63)) - 1ull) : ~0ull;

  for (int64_t row = blockIdx.x; row < a.k; row += gridDim.x) {
    const uint64_t* z = a.Z + row * W;
    // coalition size decides which polarity is cheaper to walk
    int c = 0;
    for (int64_t w0 = tid; w0 < W; w0 += 8 * kThreads) {  // eight independent loads per thread and step
      uint64_t v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int64_t w = w0 + (int64_t)q * kThreads;
        v[q] = w < W ? (z[w] & (w == W - 1 ? tail_mask : ~0ull)) : 0ull;
      }
#pragma unroll
      for (int q = 0; q < 8; ++q) c += __popcll(v[q]);
    }
    const int total = block_sum_int(c, red);
    const bool dense = 2 * (int64_t)total > a.n;
    const int step = dense ? -1 : 1;
    int* deg = (int*)rs;
    for (int i = tid; i < a.V; i += kThreads) deg[i] = dense ? (a.row_ptr[i + 1] - a.row_ptr[i] + 1) : 1;
    __syncthreads();
    // every thread walks four words at a time, so that four end-point look-ups are in flight
    for (int64_t w0 = tid; w0 < W; w0 += 4 * kThreads) {
      uint64_t bits[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int64_t w = w0 + (int64_t)q * kThreads;
        uint64_t b = 0ull;
        if (w < W) {
          b = dense ? ~z[w] : z[w];
          if (w == W - 1) b &= tail_mask;  // padding bits never name a player
        }
        bits[q] = b;
      }
      while (bits[0] | bits[1] | bits[2] | bits[3]) {
        int2 e[4];
        bool live[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          live[q] = bits[q] != 0ull;
          const int64_t p = (w0 + (int64_t)q * kThreads) * 64 + (live[q] ? __ffsll((long long)bits[q]) - 1 : 0);
          e[q] = live[q] ? a.pl[p] : make_int2(0, 0);
          bits[q] &= bits[q] - 1;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (live[q]) {
            atomicAdd(&deg[e[q].y], step);
            if (!a.directed) atomicAdd(&deg[e[q].x], step);
          }
        }
      }
    }
    __syncthreads();
    for (int i = tid; i < a.V; i += kThreads) {
      const float d = (float)deg[i];
      rs[i] = 1.0f / sqrtf(d);
    }
    __syncthreads();

    // layer 1: aggregate the shared product P = X_c W_1
    aggregate_rows(a, z, rs, a.P, a.dims[1], a.rows_out[1], a.dims[1], bufA, a.bias[0], a.L > 1, part);
    __syncthreads();
    for (int l = 2; l <= a.L; ++l) {
      aggregate_rows(a, z, rs, bufA, a.dims[l - 1], a.rows_out[l], a.dims[l - 1], bufB, nullptr, false, part);
      __syncthreads();
      transform_rows(bufB, a.rows_out[l], a.dims[l - 1], a.dims[l], a.Wl[l - 1], a.bias[l - 1], l < a.L,
                     a.bf16 != 0, bufA);
      __syncthreads();
    }
    // readout: logits of the target are bufA[0 .. d_L)
    if (tid < 64) {
      const int C = a.dims[a.L];
      float m = -INFINITY;
      for (int cidx = tid; cidx < C; cidx += 64) m = fmaxf(m, bufA[cidx]);
      for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
      float s = 0.f;
      for (int cidx = tid; cidx < C; cidx += 64) s += expf(bufA[cidx] - m);
      for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      if (tid == 0) {
        const float zc = bufA[*a.pred_ptr];
        a.y[row] = a.score == DS_SCORE_LOGIT ? zc : expf(zc - m) / s;
      }
      if (a.logits_out)
        for (int cidx = tid; cidx < C; cidx += 64) a.logits_out[row * C + cidx] = bufA[cidx];
    }
    __syncthreads();
  }
}

// ---------------- small computational graphs: one coalition per LANE ----------------
//
// When the mask row is short (n <= 2048 players) the cost of a coalition is the aggregation
// arithmetic, not the mask stream, and gathering a feature row per active edge per coalition
// keeps L2 busy instead of the ALUs. Here a workgroup takes 64 coalitions, one per lane, and every
// loop (over nodes, CSR entries, features) is uniform across the wave:
//   * the mask words of the 64 coalitions sit in LDS as zs[word][lane]; the local CSR sits in LDS too;
//   * degrees: for node v, each lane counts the set bits of its coalition among the row's
//     entries (no atomics), kept as u16 in LDS (or as d^-1/2 in a global scratch for larger graphs);
//   * layer 1, row t: H1[f][c] = sum_e P[src_e][f] * coef[e][c] with coef = bit ? d_src^-1/2 : 0 is a
//     (features x entries) . (entries x coalitions) product and runs on the matrix cores;
//   * later layers work on per-coalition operands laid out [row][feature][lane] in a global scratch: the
//     aggregation is cut into (row, 16-feature) items so that all waves stay busy; the dense transform of a
//     row, (features out x features in) . (features in x 64 coalitions), runs on the matrix cores with the
//     weight matrix staged in LDS.
// The sixteen waves of the workgroup split nodes, rows and items among them (same 64 coalitions) and
// meet at barriers between the stages.
constexpr int kBW = 32;        // mask words per coalition held in LDS (at least; more for wider masks, see the layout)
constexpr int kBWMax = 192;    // ... up to this many (12,288 players) when the rest of the LDS budget allows
constexpr int kWBufFloats = 4096;  // the workgroup's staging buffer in LDS: weight-matrix chunks of the dense transforms, and
                                   // the 64 x 64 tile in which the waves add up a shared row of layer 1
// entries per matrix-core batch of layer 1: short rows (graphs whose masks fit on chip: 15 entries a row on the
// 1,010-player config) lose less to a partly filled batch with two (0.34 -> 0.27 ms there); the long shared rows of the
// external-input mode want four entries' loads in flight (8: 14.9 ms, 4: 14.1 ms, 2: 16.2 ms on the 10^6-player config)
template <bool EXT> constexpr int stage_rows() { return EXT ? 4 : 2; }
// Waves that share the 64 coalitions of a workgroup. With the masks on chip only one workgroup fits a compute unit's LDS
// and the stages are latency chains per wave, so sixteen waves shorten them (against eight: 0.39 -> 0.32 ms on 1,010
// players, 4.1 -> 2.4 ms on 9,647). With external inputs the time is the long shared rows of layer 1, whose loop holds 64
// accumulator registers: sixteen waves leave a wave 128 registers and the loop spills, eight keep it in registers
// (config 4: 14.1 -> 13.1 ms). External inputs in pairs keep only the stored members' entry bits in LDS (half the
// bytes), so that two workgroups of four waves fit a compute unit, registers unspilled, and one's barriers and loads
// overlap the other's matrix-core work (10.2 -> 8.7 ms; three workgroups of 168 registers: 9.3 ms).
constexpr int kExtPairedThreads = 256;
template <bool EXT, bool PAIRED = false> constexpr int batched_threads() { return EXT ? (PAIRED ? kExtPairedThreads : 512) : 1024; }
constexpr int kDegLdsMaxNodes = 640;  // degrees as u16[V][64] in LDS up to this many nodes (80 KB)

struct BatchedArgs {
  EvalArgs e;
  float* scratch;          // per workgroup: rs[V][64] (if not in LDS) | bufA | bufB | q[waves][dmax][64]
  int64_t scratch_stride;  // floats per workgroup
  int64_t rs_floats, a_floats, b_floats, q_floats;  // region sizes (floats, already x64); then waves x 64 x 64
                                                    // floats of partial sums (rows shared by all waves)
  int32_t csr_lds_offset;  // byte offset of the LDS copy of the local CSR (if used)
  int32_t zs_words;        // mask words per coalition reserved in LDS (>= W)
  // external-input mode (long mask rows): degrees and entry bits as the streaming kernel wrote them, one record
  // per complementary pair (ext_paired: lanes 0..31 take the pairs' stored members, lanes 32..63 their
  // complements) or per row
  const uint16_t* ext_deg;
  const uint32_t* ext_bits;   // [record][eb_stride]: bit r = mask bit of the needed player of rank r
  const uint32_t* fdeg2;      // [V]: deg_full(v) + 2
  const int32_t* erank;       // [E_need]: rank of the player of CSR entry e among the needed players
  int64_t eb_stride;
  int32_t ext_paired, eb_words;
  int32_t ext_lr;  // ext_deg is [group of 2^ext_lr records][node][record of the group]
};

// One wave's 64 x 64 (feature x coalition) result tile of a first-layer row: accumulator register i of lane l is
// [feature 8*(i/4) + 4*(l/32) + i%4][coalition l%32]; `out` points at this lane's feature 4*(l/32) and coalition l%32.
template <bool GENERAL>
__device__ __forceinline__ void store_layer1_tile(const float16_t (&acc)[2][2], float* out, float sc0, float sc1, bool relu,
                                                  const float* bias, int fl, int d1) {
#pragma unroll
  for (int ft = 0; ft < 2; ++ft)
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int fo = ft * 32 + 8 * (i / 4) + (i % 4);
        if (!GENERAL || fl + fo < d1) {
          float v = (nb ? sc1 : sc0) * acc[ft][nb][i];
          if (GENERAL && bias) v += bias[fl + fo];
          out[fo * 64 + nb * 32] = relu ? fmaxf(v, 0.f) : v;
        }
      }
}

// zeros in place of a layer's bias vector when it has none (layer widths are at most 4096)
__device__ const float zero_bias[4096] = {};

// The per-coalition dense transform of the one-coalition-per-lane kernel ("Distributed Model Prediction", the
// |V_c| d^2 term): out[t][j][c] = act( sum_f W[f][j] q[t][f][c] + b[j] ) is, for
// every row t, a (features out x features in) . (features in x coalitions) product and runs on the matrix
// cores. A wave takes (row, 32 output features, 32 coalitions); with v_mfma_f32_32x32x2f32 lane l supplies
// W[f + l/32][j0 + l%32] (from the LDS copy of W that the workgroup stages, in row chunks if W is large) and
// q[t][f + l/32][c0 + l%32], a coalesced load in the [row][feature][coalition] layout. In the bf16
// configuration both operands are already rounded to bfloat16 (q where the aggregation stored it, W where it is
// staged) and v_mfma_f32_32x32x8bf16_1k accumulates in fp32.
template <int kBThreads>
__device__ __forceinline__ void transform_coalitions(const float* qall, float* nxt, float* Ws, const float* Wg,
                                                  const float* bias, int rows, int din, int dout, bool relu, bool isbf) {
  constexpr int kBWaves = kBThreads / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cap = kWBufFloats;
  int FB = cap / dout;
  if (FB > din) FB = din;
  if (FB < din && FB > 8) FB &= ~7;  // whole matrix-core steps per chunk
  const bool single = FB == din;
  const int jt = (dout + 31) / 32;
  const int items = rows * jt * 2;
  const int nit = (items + kBWaves - 1) / kBWaves;
  const int half = lane >> 5, r = lane & 31;
  const float* const bl = bias ? bias : zero_bias;
  for (int it = 0; it < nit; ++it) {
    const int item = it * kBWaves + wave;
    const bool live = item < items;
    const int t = live ? item / (2 * jt) : 0;
    const int rem = live ? item - t * 2 * jt : 0;
    const int j0 = (rem >> 1) * 32, c0 = (rem & 1) * 32;
    const bool jok = j0 + r < dout;
    float16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    const float* qp = qall + (size_t)t * din * 64 + c0 + r;
    for (int fb0 = 0; fb0 < din; fb0 += FB) {
      const int fcnt = din - fb0 < FB ? din - fb0 : FB;
      if (!(single && it > 0)) {
        __syncthreads();
        for (int i = tid; i < fcnt * dout; i += kBThreads) {
          const float wv = Wg[(size_t)fb0 * dout + i];
          Ws[i] = isbf ? bf16_round(wv) : wv;
        }
        __syncthreads();
      }
      if (live) {
        const float* wp = Ws + (jok ? j0 + r : 0);
        // 32 input features per step: their sixteen operand loads are in flight together
        for (int fb = 0; fb < fcnt; fb += 32) {
          float xa[4][4], xb[4][4];
#pragma unroll
          for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int f = fb + 8 * s + (isbf ? 4 * half + u : 2 * u + half);
              const bool ok = f < fcnt;
              xa[s][u] = (ok && jok) ? wp[f * dout] : 0.f;
              xb[s][u] = ok ? qp[(size_t)(fb0 + f) * 64] : 0.f;
            }
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            if (fb + 8 * s >= fcnt) break;
            if (isbf) {
              short4_t av, bv;
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                av[u] = (short)(__float_as_uint(xa[s][u]) >> 16);
                bv[u] = (short)(__float_as_uint(xb[s][u]) >> 16);
              }
              acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(av, bv, acc, 0, 0, 0);
            } else {
#pragma unroll
              for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[s][u], xb[s][u], acc, 0, 0, 0);
            }
          }
        }
      }
    }
    if (live) {
      // accumulator register i of lane l is out[feature j0 + 8*(i/4) + 4*(l/32) + i%4][coalition c0 + l%32]
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int j = j0 + 8 * (i / 4) + 4 * half + (i % 4);
        if (j < dout) {
          const float v = acc[i] + bl[j];
          nxt[((size_t)t * dout + j) * 64 + c0 + r] = relu ? fmaxf(v, 0.f) : v;
        }
      }
    }
  }
}

constexpr int kSharedRow = 256;  // a row with more entries than this is shared by all waves of the workgroup

// PAIRED (external inputs only): the records are complementary pairs and the first layer's coefficients are formed by
// the lanes that feed them to the matrix cores (see there)
template <bool DEG_LDS, bool CSR_LDS, bool EXT, bool PAIRED = false>
__global__ __launch_bounds__((batched_threads<EXT, PAIRED>()), (EXT && PAIRED ? 2 : 1)) void masked_gcn_eval_batched_kernel(BatchedArgs b) {
  const EvalArgs& a = b.e;
  constexpr int kBThreads = batched_threads<EXT, PAIRED>(), kBWaves = kBThreads / 64;
  constexpr int kStageRows = stage_rows<EXT>();
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  // LDS: zs[zs_words][64] u64 | staging buffer f32[4096] | deg[V][64] u16 (optional) | local CSR (optional)
  uint64_t* zs = (uint64_t*)smem_raw;
  const uint32_t* ebs = (const uint32_t*)smem_raw;  // EXT: entry bits as ebs[word][lane]
  float* stage_all = (float*)(smem_raw + (size_t)b.zs_words * 64 * 8);
  unsigned short* degs = (unsigned short*)(smem_raw + (size_t)b.zs_words * 64 * 8 + kWBufFloats * 4);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t *g_rp = a.row_ptr, *g_col = a.col, *g_eid = a.eid;
  if (CSR_LDS) {  // the graph structure is read many times per coalition block: keep it on chip
    const int nnz = a.row_ptr[a.V];
    int32_t* base = (int32_t*)(smem_raw + b.csr_lds_offset);
    int32_t* l_rp = base;
    int32_t* l_col = l_rp + ((a.V + 1 + 3) & ~3);
    int32_t* l_eid = l_col + ((nnz + 3) & ~3);
    for (int i = tid; i <= a.V; i += kBThreads) l_rp[i] = a.row_ptr[i];
    for (int i = tid; i < nnz; i += kBThreads) {
      l_col[i] = a.col[i];
      l_eid[i] = a.eid[i];
    }
    g_rp = l_rp;
    g_col = l_col;
    g_eid = l_eid;
  }
  const int32_t* const rp_ = g_rp;
  const int32_t* const col_ = g_col;
  const int32_t* const eid_ = g_eid;
  float* S = b.scratch + (size_t)blockIdx.x * b.scratch_stride;
  float* rs = S;
  float* bufA = rs + b.rs_floats;
  float* bufB = bufA + b.a_floats;
  const int W = (int)a.W;
  const uint64_t tail_mask = (a.n & 63) ? ((1ull << (a.n & 63)) - 1ull) : ~0ull;
  const int64_t blocks = (a.k + 63) / 64;

  const uint16_t* ext_deg_lane = nullptr;  // EXT: this lane's record in its group's block of the degrees
  int ext_member = 0;
  auto rs_of = [&](int v) -> float {
    if (EXT) {
      // the complement: d'(v) = deg_full(v) + 2 - d(v). The node is the same in every lane: the full degree comes by
      // a scalar load (no vector register, no branch on the lane's member that would hold its load back)
      typedef const __attribute__((address_space(4))) uint32_t* scalar_u32_ptr;
      const int vs = __builtin_amdgcn_readfirstlane(v);
      const int f = (int)((scalar_u32_ptr)b.fdeg2)[vs];
      const int d = ext_deg_lane[(size_t)vs << b.ext_lr];
      return __frsqrt_rn((float)(ext_member ? f - d : d));
    }
    if (DEG_LDS) return __frsqrt_rn((float)degs[v * 64 + lane]);
    return rs[(size_t)v * 64 + lane];
  };
  auto bit_of = [&](int p) -> bool { return (zs[(p >> 6) * 64 + lane] >> (p & 63)) & 1ull; };
  // mask bit of CSR entry e (of a row layer 1 produces) in this lane's coalition
  // (x: the player of the entry, or, with external inputs, the rank of that player among the needed ones)
  auto entry_bit = [&](int x) -> bool {
    // (pairs: only the stored members' words are kept, [word][pair]; the complement's bit is the inverted one)
    if (EXT && PAIRED) return (((ebs[(x >> 5) * 32 + (lane & 31)] >> (x & 31)) & 1u) ^ (uint32_t)(lane >> 5)) != 0u;
    if (EXT) return (ebs[(x >> 5) * 64 + lane] >> (x & 31)) & 1u;
    return bit_of(x);
  };
  const int32_t* const key_ = EXT ? b.erank : eid_;  // per CSR entry: what entry_bit takes

  for (int64_t blk = blockIdx.x; blk < blocks; blk += gridDim.x) {
    // EXT and paired records: lanes 0..31 are the stored members of 32 pairs, lanes 32..63 their complements
    const int member = (EXT && b.ext_paired) ? (lane >> 5) : 0;
    const int64_t rec = (EXT && b.ext_paired) ? blk * 32 + (lane & 31) : blk * 64 + lane;
    const int64_t row = (EXT && b.ext_paired) ? 2 * rec + member : rec;
    const bool valid = row < a.k;
    __syncthreads();
    if (!EXT) {
      for (int w = wave; w < W; w += kBWaves) {
        uint64_t word = valid ? a.Z[row * W + w] : 0ull;
        if (w == W - 1) word &= tail_mask;
        zs[w * 64 + lane] = word;
      }
      __syncthreads();
      // degrees: node v's entries are fetched 64 at a time by the lanes and broadcast one by one
      for (int v = wave; v < a.V; v += kBWaves) {
        const int e0 = rp_[v], e1 = rp_[v + 1];
        int cnt = 1;
        for (int eb = e0; eb < e1; eb += 64) {
          const int m = e1 - eb < 64 ? e1 - eb : 64;
          const int pv = lane < m ? eid_[eb + lane] : 0;
          for (int i = 0; i < m; ++i) cnt += bit_of(readlane_i(pv, i)) ? 1 : 0;
        }
        if (DEG_LDS) degs[v * 64 + lane] = (unsigned short)cnt;
        else rs[(size_t)v * 64 + lane] = 1.0f / sqrtf((float)cnt);
      }
    } else {
      // entry bits of this lane's record (complemented for the second member; bits past the last entry are
      // never looked at)
      uint32_t* ebw = (uint32_t*)smem_raw;
      for (int j = wave; j < b.eb_words; j += kBWaves) {
        uint32_t wd = valid ? b.ext_bits[rec * b.eb_stride + j] : 0u;
        if (PAIRED) {
          if (lane < 32) ebw[j * 32 + lane] = wd;
        } else {
          ebw[j * 64 + lane] = member ? ~wd : wd;
        }
      }
      ext_member = member;
      ext_deg_lane = b.ext_deg + (((size_t)(rec >> b.ext_lr) * a.V) << b.ext_lr) + (rec & ((1 << b.ext_lr) - 1));
    }
    __syncthreads();

    // layer 1 on the matrix cores: for row t, H1[f][c] = sum_e P[src_e][f] * coef[e][c] is a product
    // (features x entries) . (entries x coalitions). With v_mfma_f32_32x32x2f32 lane l supplies
    // A[m = l%32][k = l/32] = P[src of entry 2q + l/32][feature tile + l%32] (a plain coalesced
    // load, nothing is broadcast) and B[k = l/32][n = l%32] = coefficient of entry 2q + l/32 for
    // coalition n, which lives in another lane's register and comes over with one cross-half
    // shuffle per entry pair. The accumulator holds D[feature][coalition], so its stores are
    // 128-byte runs of consecutive coalitions.
    {
      const int d1 = a.dims[1];
      const bool relu = a.L > 1;
      const int half = lane >> 5, l32 = lane & 31;
      const float* const bias1 = a.bias[0] ? a.bias[0] : zero_bias;
      const int rows1 = a.rows_out[1];
      // One loop over the rows layer 1 produces. A row of ordinary length belongs to one wave (round-robin). A long
      // row (a hub within L-1 hops of the target) is shared: the waves split its entries, leave their partial
      // tiles in the workgroup's scratch and add them up in wave order (a fixed order: results do not depend on
      // timing).
      int ordinary = 0;
      for (int t = 0; t < rows1; ++t) {
        const int e0 = rp_[t], e1 = rp_[t + 1];  // entry e1 stands for the self-loop
        const bool shared = e1 - e0 > kSharedRow;  // the same for every wave
        if (!shared && (ordinary++ % kBWaves) != wave) continue;
        int s0 = e0, s1 = e1 + 1;
        if (shared) {
          int per = (e1 - e0 + 1 + kBWaves - 1) / kBWaves;
          per = (per + kStageRows - 1) / kStageRows * kStageRows;
          s0 = e0 + wave * per;
          s1 = s0 + per;
          if (s0 > e1 + 1) s0 = e1 + 1;
          if (s1 > e1 + 1) s1 = e1 + 1;
        }
        const float rst = rs_of(t);
        const float rst_sw = __shfl_xor(rst, 32, 64);
        for (int f0 = 0; f0 < d1; f0 += 64) {
          float16_t acc[2][2];  // [feature tile][coalition half]
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            acc[0][0][i] = 0.f; acc[0][1][i] = 0.f; acc[1][0][i] = 0.f; acc[1][1][i] = 0.f;
          }
          int pv_next = 0, sv_next = t;  // sources and keys of the step's entries, fetched one step ahead
          if (lane < kStageRows && s0 + lane < s1 && s0 + lane < e1) {
            pv_next = key_[s0 + lane];
            sv_next = col_[s0 + lane];
          }
          if (EXT && PAIRED && e1 > e0) {
            // A row's (or, of a shared row, this wave's) entries, two steps deep: the keys of step j + 2 and the operands of step j + 1 (rows of P, the
            // pair's degree, the source's full degree) are requested before the matrix cores get step j. Every load of the
            // loop is issued unconditionally (indices clamped into the row, which has at least one entry), so
            // that the wait before a step's operands is a count of younger loads and not a wait for all of them.
            constexpr int SRP = 8;   // entries per step here
            struct Ops {
              float av[SRP / 2][2];
              int d[SRP / 2], f[SRP / 2], p[SRP / 2];
            };
            auto load_keys = [&](int eb, int& pk, int& sk) {
              const int e = eb + (lane < SRP ? lane : 0);
              const bool real = e < s1 && e < e1;
              const int ec = real ? e : e1 - 1;
              const int k_ = key_[ec], c_ = col_[ec];
              pk = real ? k_ : 0;
              sk = real ? c_ : t;
            };
            auto load_ops = [&](Ops& o, int pk, int sk) {
#pragma unroll
              for (int q = 0; q < SRP / 2; ++q) {
                const int src = half ? readlane_i(sk, 2 * q + 1) : readlane_i(sk, 2 * q);
                o.p[q] = half ? readlane_i(pk, 2 * q + 1) : readlane_i(pk, 2 * q);
                const float* pr = a.P + (size_t)src * d1 + f0;
                o.av[q][0] = pr[f0 + l32 < d1 ? l32 : 0];
                o.av[q][1] = pr[f0 + 32 + l32 < d1 ? 32 + l32 : 0];
                o.d[q] = ext_deg_lane[(size_t)src << b.ext_lr];
                o.f[q] = (int)b.fdeg2[src];
              }
            };
            const bool fok0 = f0 + l32 < d1, fok1 = f0 + 32 + l32 < d1;
            Ops cur, nxt;
            int pk1, sk1;
            load_keys(s0, pk1, sk1);
            load_ops(cur, pk1, sk1);
            load_keys(s0 + SRP, pk1, sk1);
            for (int eb = s0; eb < s1; eb += SRP) {
              const int cnt = s1 - eb < SRP ? s1 - eb : SRP;
              load_ops(nxt, pk1, sk1);
              load_keys(eb + 2 * SRP, pk1, sk1);
#pragma unroll
              for (int q = 0; q < SRP / 2; ++q) {
                const int ei = 2 * q + half, p = cur.p[q];
                const bool ok = ei < cnt, self = eb + ei == e1;
                const bool bit = (ebs[(p >> 5) * 32 + l32] >> (p & 31)) & 1u;
                const float b0 = (ok && (self || bit)) ? __frsqrt_rn((float)cur.d[q]) : 0.f;              // the members
                const float b1 = (ok && (self || !bit)) ? __frsqrt_rn((float)(cur.f[q] - cur.d[q])) : 0.f;  // the complements
                const float a0 = (ok && fok0) ? cur.av[q][0] : 0.f, a1 = (ok && fok1) ? cur.av[q][1] : 0.f;
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
              }
              cur = nxt;
            }
          } else
          for (int eb = s0; eb < s1; eb += kStageRows) {
            const int cnt = s1 - eb < kStageRows ? s1 - eb : kStageRows;
            const int pv = pv_next, sv = sv_next;
            pv_next = 0;
            sv_next = t;
            if (lane < kStageRows && eb + kStageRows + lane < s1 && eb + kStageRows + lane < e1) {
              pv_next = key_[eb + kStageRows + lane];
              sv_next = col_[eb + kStageRows + lane];
            }
            float av[kStageRows / 2][2];
#pragma unroll
            for (int q = 0; q < kStageRows / 2; ++q) {
              const int s0q = readlane_i(sv, 2 * q), s1q = readlane_i(sv, 2 * q + 1);
              const int src = half ? s1q : s0q;
              const bool ok = 2 * q + half < cnt;
              const float* pr = a.P + (size_t)src * d1 + f0 + l32;
              av[q][0] = (ok && f0 + l32 < d1) ? pr[0] : 0.f;
              av[q][1] = (ok && f0 + 32 + l32 < d1) ? pr[32] : 0.f;
            }
            if (EXT && PAIRED) {
              // Lane (half, j) feeds the matrix cores the coefficients of entry 2q + half for coalition j (the stored
              // member of pair j) and coalition 32 + j (its complement): both come from one degree of the source and one
              // bit of the member's row, which this lane reads itself -- no value crosses lanes, and an entry costs one
              // degree load for the pair instead of one per member.
              float b0v[kStageRows / 2], b1v[kStageRows / 2];
#pragma unroll
              for (int q = 0; q < kStageRows / 2; ++q) {
                const int ei = 2 * q + half;
                const int p = half ? readlane_i(pv, 2 * q + 1) : readlane_i(pv, 2 * q);
                const int src = half ? readlane_i(sv, 2 * q + 1) : readlane_i(sv, 2 * q);
                const bool ok = ei < cnt, self = eb + ei == e1;
                const bool bit = (ebs[(p >> 5) * 32 + l32] >> (p & 31)) & 1u;
                const int d = ext_deg_lane[(size_t)src << b.ext_lr];
                const int f = (int)b.fdeg2[src];
                b0v[q] = (ok && (self || bit)) ? __frsqrt_rn((float)d) : 0.f;         // coalitions 0..31: the members
                b1v[q] = (ok && (self || !bit)) ? __frsqrt_rn((float)(f - d)) : 0.f;  // coalitions 32..63: the complements
              }
#pragma unroll
              for (int q = 0; q < kStageRows / 2; ++q) {
                if (2 * q < cnt) {
                  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][0], b0v[q], acc[0][0], 0, 0, 0);
                  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][0], b1v[q], acc[0][1], 0, 0, 0);
                  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][1], b0v[q], acc[1][0], 0, 0, 0);
                  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][1], b1v[q], acc[1][1], 0, 0, 0);
                }
              }
            } else if (!EXT) {
              // the same without external inputs: lane (half, j) takes the bits of coalitions j and 32 + j from their
              // mask words and the two degrees from where this kernel keeps them
              float b0v[kStageRows / 2], b1v[kStageRows / 2];
#pragma unroll
              for (int q = 0; q < kStageRows / 2; ++q) {
                const int ei = 2 * q + half;
                const int p = half ? readlane_i(pv, 2 * q + 1) : readlane_i(pv, 2 * q);
                const int src = half ? readlane_i(sv, 2 * q + 1) : readlane_i(sv, 2 * q);
                const bool ok = ei < cnt, self = eb + ei == e1;
                const uint64_t* zw = zs + (p >> 6) * 64 + l32;
                const bool bit0 = (zw[0] >> (p & 63)) & 1ull, bit1 = (zw[32] >> (p & 63)) & 1ull;
                float r0, r1;
                if (DEG_LDS) {
                  r0 = __frsqrt_rn((float)degs[src * 64 + l32]);
                  r1 = __frsqrt_rn((float)degs[src * 64 + 32 + l32]);
                } else {
                  r0 = rs[(size_t)src * 64 + l32];
                  r1 = rs[(size_t)src * 64 + 32 + l32];
                }
                b0v[q] = (ok && (self || bit0)) ? r0 : 0.f;
                b1v[q] = (ok && (self || bit1)) ? r1 : 0.f;
              }
#pragma unroll
              for (int q = 0; q < kStageRows / 2; ++q) {
                if (2 * q < cnt) {
                  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][0], b0v[q], acc[0][0], 0, 0, 0);
                  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][0], b1v[q], acc[0][1], 0, 0, 0);
                  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][1], b0v[q], acc[1][0], 0, 0, 0);
                  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][1], b1v[q], acc[1][1], 0, 0, 0);
                }
              }
            } else {
            float coef[kStageRows];
#pragma unroll
            for (int i = 0; i < kStageRows; ++i) {
              coef[i] = 0.f;
              if (i < cnt) {
                const bool self = eb + i == e1;
                const int p = readlane_i(pv, i), src = readlane_i(sv, i);
                const float r = rs_of(src);
                coef[i] = (self || entry_bit(p)) ? r : 0.f;
              }
            }
#pragma unroll
            for (int q = 0; q < kStageRows / 2; ++q) {
              if (2 * q < cnt) {
                const float x = coef[2 * q], y = coef[2 * q + 1];
                const float xs = __shfl_xor(x, 32, 64), ys = __shfl_xor(y, 32, 64);
                const float b0 = half ? ys : x;  // coalitions 0..31
                const float b1 = half ? y : xs;  // coalitions 32..63
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][0], b0, acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][0], b1, acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][1], b0, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q][1], b1, acc[1][1], 0, 0, 0);
              }
            }
            }
          }
          // accumulator register i of lane l is D[feature 8*(i/4) + 4*(l/32) + i%4][coalition l%32]
          if (!shared) {
            // a full tile without a bias (the usual case) is stored without a test or a load per element
            const int fl = f0 + 4 * half;
            float* out = bufA + ((size_t)t * d1 + fl) * 64 + l32;
            const float sc0 = half ? rst_sw : rst, sc1 = half ? rst : rst_sw;  // d^-1/2 of row t in coalitions l32, 32 + l32
            if (a.bias[0] == nullptr && f0 + 64 <= d1)
              store_layer1_tile<false>(acc, out, sc0, sc1, relu, nullptr, fl, d1);
            else
              store_layer1_tile<true>(acc, out, sc0, sc1, relu, a.bias[0], fl, d1);
          } else {
            // the waves add their tiles into one LDS tile, one wave at a time in wave order
            float* tl = stage_all + (4 * half) * 64 + l32;  // the staging area is idle during layer 1
            for (int w = 0; w < kBWaves; ++w) {
              if (wave == w) {
#pragma unroll
                for (int ft = 0; ft < 2; ++ft)
#pragma unroll
                  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                      float* dst = tl + (ft * 32 + 8 * (i / 4) + (i % 4)) * 64 + nb * 32;
                      *dst = w == 0 ? acc[ft][nb][i] : *dst + acc[ft][nb][i];
                    }
              }
              __syncthreads();
            }
#pragma unroll 1
            for (int j = 0; j < 4096 / kBThreads; ++j) {
              const int idx = tid + j * kBThreads;  // feature idx / 64 of the tile, coalition idx % 64 == lane
              const int fr = f0 + (idx >> 6);
              if (fr < d1) {
                const float v = rst * stage_all[idx] + bias1[fr];
                bufA[((size_t)t * d1 + fr) * 64 + lane] = relu ? fmaxf(v, 0.f) : v;
              }
            }
            __syncthreads();
          }
        }
      }
    }
    __syncthreads();

    float* cur = bufA;
    float* nxt = bufB;
    float* qall = bufB + b.b_floats;  // q[row][feature][lane] of the layer in flight
    for (int l = 2; l <= a.L; ++l) {
      const int din = a.dims[l - 1], dout = a.dims[l];
      const bool relu = l < a.L;
      const int rows = a.rows_out[l];
      // These layers have few rows but long dependent chains, so the work is cut into
      // (row, 16-feature slice) items spread over all waves, four entries in flight per step.
      // phase A: q[t][f] = rs_t * ( sum_active rs_src H[src][f] + rs_t H[t][f] )
      const int fch = (din + 15) / 16;
      for (int item = wave; item < rows * fch; item += kBWaves) {
        const int t = item / fch, f0 = (item - t * fch) * 16;
        const int e0 = rp_[t], e1 = rp_[t + 1];
        const float rst = rs_of(t);
        float acc[16];
#pragma unroll
        for (int f = 0; f < 16; ++f) acc[f] = 0.f;
        for (int eb = e0; eb <= e1; eb += 4) {  // entry e1 stands for the self-loop
          float c[4];
          const float* hp[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int e = eb + u;
            int src = t;
            c[u] = 0.f;
            if (e < e1) {
              src = col_[e];
              c[u] = entry_bit(key_[e]) ? rs_of(src) : 0.f;
            } else if (e == e1) {
              c[u] = rst;
            }
            hp[u] = cur + ((size_t)src * din + f0) * 64 + lane;
          }
          float hv[4][16];
#pragma unroll
          for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int f = 0; f < 16; ++f) hv[u][f] = (f0 + f < din) ? hp[u][(size_t)f * 64] : 0.f;
#pragma unroll
          for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int f = 0; f < 16; ++f) acc[f] += c[u] * hv[u][f];
        }
#pragma unroll
        for (int f = 0; f < 16; ++f)
          if (f0 + f < din) {
            const float q = rst * acc[f];
            qall[((size_t)t * din + f0 + f) * 64 + lane] = a.bf16 ? bf16_round(q) : q;
          }
      }
      __syncthreads();
      transform_coalitions<kBThreads>(qall, nxt, stage_all, a.Wl[l - 1], a.bias[l - 1], rows, din, dout, relu, a.bf16 != 0);
      __syncthreads();
      float* tmp = cur; cur = nxt; nxt = tmp;
    }

    // readout: logits of the target are cur[c][lane], c < d_L (row 0)
    if (wave == 0 && valid) {
      const int C = a.dims[a.L];
      float m = -INFINITY;
      for (int c = 0; c < C; ++c) m = fmaxf(m, cur[(size_t)c * 64 + lane]);
      float sum = 0.f;
      for (int c = 0; c < C; ++c) sum += expf(cur[(size_t)c * 64 + lane] - m);
      const float zc = cur[(size_t)(*a.pred_ptr) * 64 + lane];
      a.y[row] = a.score == DS_SCORE_LOGIT ? zc : expf(zc - m) / sum;
      if (a.logits_out)
        for (int c = 0; c < C; ++c) a.logits_out[row * C + c] = cur[(size_t)c * 64 + lane];
    }
  }
}

// ---------------- large computational graphs: the mask matrix is streamed once ----------------
//
// When a mask row is long (more than 12,288 players) everything a coalition's evaluation needs from its
// row is (a) the degree of every node and (b) the bits of the CSR entries of the rows layer 1 has to
// produce (the nodes within L-1 hops of the target; their entries are a prefix of the local CSR). A first
// kernel streams the rows and reduces each to exactly that, a few KB per coalition; the layers then run
// on 64 coalitions per workgroup from those compact arrays (the one-coalition-per-lane kernel in its
// external-input mode), with the shared first product on the matrix cores.
//
// Complementary pairs (rows 2r, 2r+1 as the sampler writes them): only row 2r, the smaller member, is read.
// Its complement has d'(v) = deg_full(v) + 2 - d(v) and the opposite entry bits, which the second kernel
// derives itself, so the stream is half of the mask matrix.
struct StreamArgs {
  int32_t V, n, directed, E_need;
  int32_t lr;         // log2 of the rows a workgroup takes together (1..3)
  int32_t cnt_words;  // u32 words of the group's packed 16-bit counters: V x R / 2 (node-major: a node's R counters are consecutive)
  int32_t slots;      // records per block of the transposed degree array: 32 (pairs) or 64 (single rows)
  int32_t size_step;  // row r's coalition size is sizes[r * size_step]
  int64_t W, rows, row_stride;  // rows handled by this launch; words between consecutive handled rows
  const uint64_t* Z;
  const int32_t* sizes;
  const uint32_t* pab;          // [n] end points of player p as local ids: a in the low, b in the high 16 bits
  const uint64_t* wsplit;       // [W] bit j: player 64w + j (j > 0) has another first end point than the player before it
  const int32_t* wfirst;        // [W] first end point of player 64w
  const int32_t* row_ptr;
  const uint64_t* nmask;        // [W] bits of the players whose CSR entries layer 1 reads ("needed" players)
  const int32_t* nbase;         // [W] number of needed players before word w: a needed player's rank = nbase + rank in word
  const int32_t* need_range;    // [2]: the words that hold needed players lie in [need_range[0], need_range[1])
  int32_t eb_words;             // u32 words of a row's needed bits (rank order)
  uint16_t* deg_out;            // [group][V][R]: d(v) = 1 + active entries of row v, record = group * R + row of the group
  uint32_t* ebits_out;          // [rows][eb_stride] bit r = mask bit of the needed player of rank r
  int64_t eb_stride;
  // the players of sparse rows as lists (the sampler writes them beside the mask rows), or null: row r's players are
  // list[list_offset[r] .. + sizes[r]) in any order when list_offset[r] >= 0; such a row's bits are not read at all
  const uint32_t* list;
  const int64_t* list_offset;
};

// (256 threads per workgroup: a wave is the 64 players of one mask word)
__global__ void pack_endpoints_kernel(const int2* pl, int64_t n, uint32_t* pab, unsigned long long* wsplit, int32_t* wfirst) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  bool starts = false;
  if (p < n) {
    const int2 e = pl[p];
    pab[p] = (uint32_t)e.x | ((uint32_t)e.y << 16);
    if ((p & 63) == 0) wfirst[p >> 6] = e.x;
    else starts = pl[p - 1].x != e.x;
  }
  const unsigned long long m = __ballot(starts);
  if ((threadIdx.x & 63) == 0 && p < n) wsplit[p >> 6] = m;
}

// coalition size of every handled row, one wave per row (only when the caller has no sizes at hand)
__global__ __launch_bounds__(kThreads) void mask_row_sizes_kernel(const uint64_t* Z, int64_t rows, int64_t row_stride, int64_t W,
                                                                int32_t* sizes) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6, nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t r = wave; r < rows; r += nwaves) {
    const uint64_t* z = Z + r * row_stride;
    int c = 0;
    for (int64_t w = lane; w < W; w += 64) c += __popcll(z[w]);  // padding bits are zero
    for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
    if (lane == 0) sizes[r] = c;
  }
}

// needed players: mark, (scan of the per-word counts on the host side), rank of every needed CSR entry's player
__global__ void full_degree_kernel(const int32_t* row_ptr, int V, uint32_t* fdeg2) {
  const int v = blockIdx.x * blockDim.x + threadIdx.x;
  if (v < V) fdeg2[v] = (uint32_t)(row_ptr[v + 1] - row_ptr[v] + 2);
}
__global__ void zero_u64_kernel(uint64_t* x, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) x[i] = 0ull;
}
__global__ void need_mark_kernel(const int32_t* eid, int E_need, unsigned long long* nmask) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E_need) return;
  const int p = eid[e];
  atomicOr(&nmask[p >> 6], 1ull << (p & 63));
}
__global__ void need_count_kernel(const uint64_t* nmask, int64_t W, int32_t* cnt) {
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w < W) cnt[w] = __popcll(nmask[w]);
}
__global__ void need_range_kernel(const uint64_t* nmask, int64_t W, int32_t* range) {
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w < W && nmask[w] != 0ull) {
    atomicMin(&range[0], (int32_t)w);
    atomicMax(&range[1], (int32_t)w + 1);
  }
}
__global__ void need_rank_kernel(const int32_t* eid, int E_need, const uint64_t* nmask, const int32_t* nbase, int32_t* erank) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= E_need) return;
  const int p = eid[e];
  erank[e] = nbase[p >> 6] + __popcll(nmask[p >> 6] & ((1ull << (p & 63)) - 1ull));
}

constexpr int kSThreads = 1024;
constexpr int kSWaves = kSThreads / 64;
constexpr int kQueueCap = 512;  // players a wave lists before it looks their end points up
constexpr int kDenseShift = 4;    // a row walks player by player (not bit by bit) from n / 16 bits to count ...
constexpr int kDenseMinBits = 64;  // ... and this many

// A workgroup of sixteen waves takes R = 2^lr consecutive rows together and counts, for every row, the set bits (or,
// when more than half are set, the cleared ones) incident to every node, with LDS atomics on 16-bit counters packed in
// pairs. The counters of eight rows of a 7,500-node computation graph fill most of a compute unit's LDS, so one
// workgroup runs per unit: sixteen waves (not eight) are what keeps enough loads in flight.
// Rows with few bits to count are walked bit by bit, a wave streaming one row 1 KB at a time; set bits are listed
// in the wave's LDS queue and their end points looked up in batches. Rows with many bits are walked player by player:
// the 64 words of a block are cut into 16-bit pieces in LDS so that a lane, holding the end points of one player of the
// word (one coalesced load for all rows of the group), gets the increments of two rows with one shift and one AND
// and adds four rows to the player's second end point with one 64-bit atomic; the first end points of consecutive
// players are equal, so they are counted by one popcount per run while a lane still holds the whole word. The
// needed players' bits are taken from the words as they pass, only in the stretch of the row that holds any.
// Degrees go out as one contiguous block per workgroup ([group][node][row]).
// inclusive prefix sum over the 64 lanes of a wave, by data-parallel-primitive moves inside the rows of 16 lanes and two
// broadcasts across them (no LDS traffic)
__device__ __forceinline__ int wave_inclusive_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false); // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false); // row_bcast:31 into rows 2 and 3
  return v;
}

template <bool PAIRED, int LR>
__global__ __launch_bounds__(kSThreads) void stream_degrees_kernel(StreamArgs a) {
  extern __shared__ uint32_t ssm[];  // V x R packed 16-bit counters, 8 mode words, the waves' player queues
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int R = 1 << LR;  // rows per workgroup
  uint32_t* cnt_all = ssm;
  int* modes = (int*)(ssm + a.cnt_words);  // bit 0: the cleared bits are walked, bit 1: player by player, bit 2: from a list
  uint32_t* queue = ssm + a.cnt_words + 8;  // kSWaves queues of kQueueCap players
  uint32_t* nb_all = queue + kSWaves * kQueueCap;       // R x eb_words needed bits
  // 16-bit counters, two rows to a u32 (row r: half r & 1 of pair r >> 1). Up to four rows (two pairs) of a node are
  // consecutive; with eight rows, rows 4..7 form a second array behind the first, so that a 64-bit atomic on the rows
  // 0..3 (or 4..7) of the nodes spreads over sixteen pairs of LDS banks instead of eight
  constexpr int lrh = LR == 3 ? 1 : LR - 1;
  const int cnt_half = LR == 3 ? a.cnt_words / 2 : 0;
  auto cnt_word = [&](uint32_t node, int pair) -> uint32_t* { return cnt_all + (pair >> 1) * cnt_half + (node << lrh) + (pair & 1); };
  auto count_one = [&](uint32_t node, int row) { atomicAdd(cnt_word(node, row >> 1), 1u << ((row & 1) << 4)); };
  const int64_t W = a.W;
  const uint64_t tail_mask = (a.n & 63) ? ((1ull << (a.n & 63)) - 1ull) : ~0ull;
  const int64_t groups = (a.rows + R - 1) / R;
  for (int64_t g = blockIdx.x; g < groups; g += gridDim.x) {
    for (int i = tid; i < a.cnt_words; i += kSThreads) cnt_all[i] = 0u;
    for (int i = tid; i < R * a.eb_words; i += kSThreads) nb_all[i] = 0u;
    if (tid < R) {
      const int64_t rr = g * R + tid;
      int mode = 0;
      if (rr < a.rows) {
        const int64_t sz = a.sizes[rr * a.size_step];
        const bool flip = !PAIRED && 2 * sz > a.n;
        const int64_t walk = flip ? a.n - sz : sz;
        mode = (flip ? 1 : 0) | (((walk << kDenseShift) >= a.n && walk >= kDenseMinBits) ? 2 : 0);
        if (PAIRED && a.list_offset != nullptr && mode == 0 && a.list_offset[rr] >= 0) mode = 4;  // its players come as a list
      }
      modes[tid] = mode;
    }
    __syncthreads();
    int any_dense = 0;
    for (int i = 0; i < R; ++i) any_dense |= modes[i] & 2;
    const int64_t need_lo = a.need_range[0], need_hi = a.need_range[1];
    // the needed players' bits of mask word `word` (true bits, word index w) of group row `row`, in rank order
    auto take_needed = [&](uint64_t word, uint64_t nm, int r0, int row) {  // r0: needed players before this word
      uint64_t x = word & nm;
      if (x == 0ull) return;
      uint32_t* nb = nb_all + (size_t)row * a.eb_words;
      if (nm == ~0ull) {  // a run of needed players (the players of a hub come one after another)
        const int sh = r0 & 31;
        atomicOr(&nb[r0 >> 5], (uint32_t)(x << sh));
        atomicOr(&nb[(r0 >> 5) + 1], (uint32_t)(x >> (32 - sh)));
        if (sh) atomicOr(&nb[(r0 >> 5) + 2], (uint32_t)(x >> (64 - sh)));
        return;
      }
      while (x) {
        const int j = __ffsll((long long)x) - 1;
        x &= x - 1;
        const int r = r0 + __popcll(nm & ((1ull << j) - 1ull));
        atomicOr(&nb[r >> 5], 1u << (r & 31));
      }
    };
    // ---- rows walked bit by bit. Looking up a player's end points right where its bit is found makes every step
    // wait for a memory round trip that serves a few bits; instead the wave first only lists the players (the bit
    // positions) in a queue of its own in LDS, and empties the queue when it is nearly full: then every lane has
    // eight independent look-ups in flight, whatever word they came from.
    // A wave streams ONE row (with fewer than eight rows to a group, a part of one): a load is 1 KB of consecutive
    // mask words, 16 bytes a lane, four loads make a step, and the next step's loads are issued before the current
    // step's words are looked at.
    {
      constexpr int wpr = kSWaves / R;   // waves that share a row
      const int qrow = __builtin_amdgcn_readfirstlane(wave / wpr), part = __builtin_amdgcn_readfirstlane(wave % wpr);
      const int64_t r = g * R + qrow;
      const int mode = modes[qrow];
      const bool active = r < a.rows && !(mode & 6);   // the same for the whole wave
      const bool flip = mode & 1;
      const uint64_t* z = a.Z + (r < a.rows ? r : 0) * a.row_stride;
      uint32_t* myq = queue + wave * kQueueCap;
      int qfill = 0;  // the same in every lane
      auto drain = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        for (int i0 = 0; i0 < qfill; i0 += 512) {
          uint32_t ent[8], e[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int idx = i0 + u * 64 + lane;
            ent[u] = idx < qfill ? myq[idx] : 0xFFFFFFFFu;
            e[u] = ent[u] != 0xFFFFFFFFu ? a.pab[ent[u]] : 0u;
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            if (ent[u] != 0xFFFFFFFFu) {
              count_one(e[u] >> 16, qrow);
              if (!a.directed) count_one(e[u] & 0xFFFFu, qrow);
            }
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        qfill = 0;
      };
      typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));
      const bool wide_ok = ((a.row_stride & 1) == 0) && (((uintptr_t)a.Z & 15) == 0);  // rows start on 16 bytes
      constexpr int kLd = 4;  // loads per step
      constexpr int wstep = kLd * wpr * 128;  // words of a row one step of its waves covers
      // first word of this lane's u-th load of the step at wc0
      auto word_of = [&](int64_t wc0, int u) -> int64_t { return wc0 + (int64_t)(u * wpr + part) * 128 + 2 * lane; };
      auto fetch = [&](int64_t wc0, u64x2 (&dst)[kLd]) {  // a step that lies wholly inside the row
#pragma unroll
        for (int u = 0; u < kLd; ++u) dst[u] = __builtin_nontemporal_load((const u64x2*)(z + word_of(wc0, u)));  // streamed once
      };
      auto fetch_checked = [&](int64_t wc0, u64x2 (&dst)[kLd]) {  // the last step, or rows that are not 16-byte aligned
#pragma unroll
        for (int u = 0; u < kLd; ++u) {
          const int64_t w = word_of(wc0, u);
          dst[u][0] = w < W ? z[w] : (flip ? ~0ull : 0ull);
          dst[u][1] = w + 1 < W ? z[w + 1] : (flip ? ~0ull : 0ull);
          if (w == W - 1) dst[u][0] = flip ? dst[u][0] | ~tail_mask : dst[u][0] & tail_mask;  // padding bits name no player
          if (w + 1 == W - 1) dst[u][1] = flip ? dst[u][1] | ~tail_mask : dst[u][1] & tail_mask;
        }
      };
      auto step = [&](int64_t wc0, const u64x2 (&v)[kLd]) {
        const bool need_here = wc0 < need_hi && wc0 + wstep > need_lo;
#pragma unroll
        for (int u = 0; u < kLd; ++u) {  // one load's 128 words at a time: at most a few hundred bits
          uint64_t t0 = v[u][0], t1 = v[u][1];
          const int64_t w = word_of(wc0, u);
          if (need_here) {  // (true bits: before the flip)
            if (w < W) take_needed(t0, a.nmask[w], a.nbase[w], qrow);
            if (w + 1 < W) take_needed(t1, a.nmask[w + 1], a.nbase[w + 1], qrow);
          }
          if (flip) {
            t0 = ~t0;
            t1 = ~t1;
          }
          uint32_t x[4] = {(uint32_t)t0, (uint32_t)(t0 >> 32), (uint32_t)t1, (uint32_t)(t1 >> 32)};
          const int c = __popc(x[0]) + __popc(x[1]) + __popc(x[2]) + __popc(x[3]);
          if (__ballot(c != 0) == 0ull) continue;
          const int incl = wave_inclusive_sum(c);
          const int total = __builtin_amdgcn_readlane(incl, 63);
          const uint32_t pb = (uint32_t)(w * 64);
          if (total > kQueueCap) {  // more bits than the queue holds at once: counted directly
            if (qfill) drain();
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              uint32_t bits = x[j];
              while (bits) {
                const uint32_t e = a.pab[pb + 32 * j + (__ffs((int)bits) - 1)];
                bits &= bits - 1;
                count_one(e >> 16, qrow);
                if (!a.directed) count_one(e & 0xFFFFu, qrow);
              }
            }
            continue;
          }
          if (qfill + total > kQueueCap) drain();
          int pos = qfill + incl - c;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            uint32_t bits = x[j];
            while (bits) {
              myq[pos++] = (pb + 32 * j) + (uint32_t)(__ffs((int)bits) - 1);
              bits &= bits - 1;
            }
          }
          qfill += total;
        }
      };
      if (active) {
        int64_t wc0 = 0;
        u64x2 cur[kLd], nxt[kLd];
        if (wide_ok && wstep < W) {
          fetch(0, cur);
          for (; wc0 + 2 * wstep < W; wc0 += wstep) {  // the step after this one lies inside the row as well
            fetch(wc0 + wstep, nxt);
            step(wc0, cur);
#pragma unroll
            for (int u = 0; u < kLd; ++u) cur[u] = nxt[u];
          }
          step(wc0, cur);
          wc0 += wstep;
        }
        for (; wc0 < W; wc0 += wstep) {
          fetch_checked(wc0, cur);
          step(wc0, cur);
        }
        if (qfill) drain();
      }
      // ---- rows whose players come as a list: 4 bytes per player instead of the n / 8 bytes of the bit row. The waves
      // of the row take 512 entries at a time, eight per lane, with the eight end-point look-ups in flight together.
      if (r < a.rows && (mode & 4)) {
        const uint32_t* lst = a.list + a.list_offset[r];
        const int s = a.sizes[r * a.size_step];
        uint32_t* nb = nb_all + (size_t)qrow * a.eb_words;
        for (int i0 = part * 512; i0 < s; i0 += wpr * 512) {
          uint32_t ent[8], e[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const int idx = i0 + u * 64 + lane;
            ent[u] = idx < s ? lst[idx] : 0xFFFFFFFFu;
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) e[u] = ent[u] < (uint32_t)a.n ? a.pab[ent[u]] : 0u;
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            if (ent[u] < (uint32_t)a.n) {
              count_one(e[u] >> 16, qrow);
              if (!a.directed) count_one(e[u] & 0xFFFFu, qrow);
              const int64_t w = ent[u] >> 6;
              if (w >= need_lo && w < need_hi) {
                const uint64_t nm = a.nmask[w];
                const int j = ent[u] & 63;
                if ((nm >> j) & 1ull) {
                  const int rk = a.nbase[w] + __popcll(nm & ((1ull << j) - 1ull));
                  atomicOr(&nb[rk >> 5], 1u << (rk & 31));
                }
              }
            }
          }
        }
      }
    }
    // ---- rows walked player by player. A wave takes a contiguous range of word columns, 64 words at a time with
    // lane = word (coalesced loads of every dense row of the group). While a lane holds its word of the R rows it
    // (a) takes the needed players' bits, (b) counts the FIRST end points: players with the same first end point
    // are consecutive, so a word is a few runs (wsplit marks where a new one starts, wfirst names the first) and a
    // run's count in a row is one popcount, (c) leaves the words in the wave's LDS area cut into 16-bit pieces, two
    // rows to a u32: [word][piece][row pair]. Then the words are walked with lane = player: a lane reads the 16 bytes
    // that hold its piece of all eight rows, and (x >> (lane & 15)) & 0x00010001 is at once the pair of 16-bit
    // increments of two rows, so one 64-bit LDS atomic adds four rows' bits to the player's SECOND end point.
    if (any_dense) {
      int dmode[8];  // per row of the group: -1 = not walked this way, else bit 0 of its mode (wave-uniform values)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int m = i < R ? __builtin_amdgcn_readfirstlane(modes[i < R ? i : 0]) : 0;
        dmode[i] = (i < R && (m & 2)) ? (m & 1) : -1;
      }
      uint32_t* stage = queue + wave * kQueueCap;  // the wave's queue is empty by now: 32 words x 4 pieces x 4 u32
      const int64_t per = ((W + kSWaves - 1) / kSWaves + 63) & ~(int64_t)63;
      const int64_t w_begin = (int64_t)__builtin_amdgcn_readfirstlane(wave) * per;
      const int64_t w_end = w_begin + per < W ? w_begin + per : W;
      uint64_t mw_next[8];
      auto load_words = [&](int64_t wb, uint64_t (&dst)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          uint64_t m = 0ull;
          if (dmode[i] >= 0 && wb + lane < w_end) m = __builtin_nontemporal_load(&a.Z[(g * R + i) * a.row_stride + wb + lane]);
          dst[i] = m;
        }
      };
      auto load_players = [&](int64_t w0, uint32_t (&dst)[8]) {  // end points of player `lane` of eight consecutive words
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int64_t p = (w0 + u) * 64 + lane;
          dst[u] = p < a.n ? a.pab[p] : 0u;
        }
      };
      // adds the packed increments inc[h] = (row 2h) | (row 2h+1) << 16 to the counters of `node`
      auto add_packed = [&](uint32_t node, const uint32_t (&inc)[4]) {
        if (R == 2) {
          if (inc[0]) atomicAdd(cnt_word(node, 0), inc[0]);
        } else {
          if (inc[0] | inc[1])
            atomicAdd((unsigned long long*)cnt_word(node, 0), (unsigned long long)inc[0] | ((unsigned long long)inc[1] << 32));
          if (R == 8 && (inc[2] | inc[3]))
            atomicAdd((unsigned long long*)cnt_word(node, 2), (unsigned long long)inc[2] | ((unsigned long long)inc[3] << 32));
        }
      };
      if (w_begin < w_end) load_words(w_begin, mw_next);
      for (int64_t wb = w_begin; wb < w_end; wb += 64) {
        const bool in = wb + lane < w_end;
        const bool need_blk = wb < need_hi && wb + 64 > need_lo;
        const uint64_t nmw = (in && need_blk) ? a.nmask[wb + lane] : 0ull;
        const int nrw = (in && need_blk) ? a.nbase[wb + lane] : 0;
        uint64_t split = (in && !a.directed) ? a.wsplit[wb + lane] : 0ull;
        uint32_t node = (in && !a.directed) ? (uint32_t)a.wfirst[wb + lane] : 0u;
        uint64_t mw[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          uint64_t m = mw_next[i];
          if (dmode[i] >= 0 && in) {
            if (need_blk) take_needed(m, nmw, nrw, i);
            if (dmode[i]) m = ~m;
            if (wb + lane == W - 1) m &= tail_mask;
          }
          mw[i] = m;
        }
        if (wb + 64 < w_end) load_words(wb + 64, mw_next);
        uint32_t e_next[8];
        load_players(wb, e_next);
        // (b) first end points
        if (!a.directed) {
          auto run_counts = [&](uint64_t seg, uint32_t (&inc)[4]) {
#pragma unroll
            for (int h = 0; h < 4; ++h) {
              inc[h] = 0u;
              if (2 * h < R) inc[h] = (uint32_t)__popcll(mw[2 * h] & seg) | ((uint32_t)__popcll(mw[2 * h + 1] & seg) << 16);
            }
          };
          const uint32_t node0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)node);
          if (__ballot(split != 0ull || node != node0 || !in) == 0ull) {
            // one run covers all 64 words (inside a hub's players): add the lanes' counts up first (at most 64 x 64 per
            // 16-bit field), one lane adds them to the counters
            uint32_t inc[4];
            run_counts(~0ull, inc);
#pragma unroll
            for (int h = 0; h < 4; ++h)
              if (2 * h < R)
                for (int o = 32; o > 0; o >>= 1) inc[h] += __shfl_xor(inc[h], o, 64);
            if (lane == 0) add_packed(node0, inc);
          } else if (in) {
            int lo = 0;
            for (;;) {
              const int hi = split ? __ffsll((long long)split) - 1 : 64;  // the run covers bits lo .. hi-1
              const uint64_t seg = (hi >= 64 ? ~0ull : ((1ull << hi) - 1ull)) & ~((1ull << lo) - 1ull);
              uint32_t inc[4];
              run_counts(seg, inc);
              add_packed(node, inc);
              if (!split) break;
              split &= split - 1;
              lo = hi;
              node = a.pab[(wb + lane) * 64 + lo] & 0xFFFFu;
            }
          }
        }
        // (c) + second end points, 32 words at a time
#pragma unroll 1
        for (int hb = 0; hb < 2; ++hb) {
          if (wb + 32 * hb >= w_end) break;
          __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
          if ((lane >> 5) == hb) {
            uint4* dst = (uint4*)stage + (lane & 31) * 4;
            const uint32_t lo0 = (uint32_t)mw[0], lo1 = (uint32_t)mw[1], lo2 = (uint32_t)mw[2], lo3 = (uint32_t)mw[3];
            const uint32_t lo4 = (uint32_t)mw[4], lo5 = (uint32_t)mw[5], lo6 = (uint32_t)mw[6], lo7 = (uint32_t)mw[7];
            const uint32_t hi0 = (uint32_t)(mw[0] >> 32), hi1 = (uint32_t)(mw[1] >> 32), hi2 = (uint32_t)(mw[2] >> 32);
            const uint32_t hi3 = (uint32_t)(mw[3] >> 32), hi4 = (uint32_t)(mw[4] >> 32), hi5 = (uint32_t)(mw[5] >> 32);
            const uint32_t hi6 = (uint32_t)(mw[6] >> 32), hi7 = (uint32_t)(mw[7] >> 32);
            // __builtin_amdgcn_perm(x, y, sel): byte k of the result is byte sel[k] of {x (bytes 4..7), y (bytes 0..3)}
            constexpr uint32_t kLow = 0x05040100u, kHigh = 0x07060302u;  // the low / high halves of y and x
            dst[0] = make_uint4(__builtin_amdgcn_perm(lo1, lo0, kLow), __builtin_amdgcn_perm(lo3, lo2, kLow),
                                __builtin_amdgcn_perm(lo5, lo4, kLow), __builtin_amdgcn_perm(lo7, lo6, kLow));
            dst[1] = make_uint4(__builtin_amdgcn_perm(lo1, lo0, kHigh), __builtin_amdgcn_perm(lo3, lo2, kHigh),
                                __builtin_amdgcn_perm(lo5, lo4, kHigh), __builtin_amdgcn_perm(lo7, lo6, kHigh));
            dst[2] = make_uint4(__builtin_amdgcn_perm(hi1, hi0, kLow), __builtin_amdgcn_perm(hi3, hi2, kLow),
                                __builtin_amdgcn_perm(hi5, hi4, kLow), __builtin_amdgcn_perm(hi7, hi6, kLow));
            dst[3] = make_uint4(__builtin_amdgcn_perm(hi1, hi0, kHigh), __builtin_amdgcn_perm(hi3, hi2, kHigh),
                                __builtin_amdgcn_perm(hi5, hi4, kHigh), __builtin_amdgcn_perm(hi7, hi6, kHigh));
          }
          __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
          const int64_t w0 = wb + 32 * hb;
          const uint4* src = (const uint4*)stage + (lane >> 4);
          const int sh = lane & 15;
          for (int j0 = 0; j0 < 32 && w0 + j0 < w_end; j0 += 8) {
            uint32_t e[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) e[u] = e_next[u];
            if (w0 + j0 + 8 < w_end && (hb == 0 || j0 + 8 < 32)) load_players(w0 + j0 + 8, e_next);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
              const uint4 x = src[(j0 + u) * 4];
              uint32_t inc[4];
              inc[0] = (x.x >> sh) & 0x00010001u;
              inc[1] = (x.y >> sh) & 0x00010001u;
              inc[2] = (x.z >> sh) & 0x00010001u;
              inc[3] = (x.w >> sh) & 0x00010001u;
              add_packed(e[u] >> 16, inc);
            }
          }
        }
      }
    }
    __syncthreads();
    // degrees: [group][node][row of the group], one contiguous block per workgroup (whole cache lines are written)
    {
      uint16_t* dst = a.deg_out + (size_t)g * a.V * R;
      for (int v = tid; v < a.V; v += kSThreads) {
        const int full1 = PAIRED ? 0 : a.row_ptr[v + 1] - a.row_ptr[v] + 1;  // (only a walk over cleared bits needs it)
        uint32_t d[R / 2];
#pragma unroll
        for (int q2 = 0; q2 < R; q2 += 2) {
          const uint32_t cw = *cnt_word((uint32_t)v, q2 >> 1);
          int c0 = cw & 0xFFFF, c1 = cw >> 16;
          if (!PAIRED) {
            if (modes[q2] & 1) c0 = full1 - 1 - c0;
            if (modes[q2 + 1] & 1) c1 = full1 - 1 - c1;
          }
          d[q2 >> 1] = (uint32_t)(c0 + 1) | ((uint32_t)(c1 + 1) << 16);
        }
        uint32_t* d32 = (uint32_t*)(dst + (size_t)v * R);
        if (R == 8) *(uint4*)d32 = make_uint4(d[0], d[1 % (R / 2)], d[2 % (R / 2)], d[3 % (R / 2)]);
        else if (R == 4) *(uint2*)d32 = make_uint2(d[0], d[1 % (R / 2)]);
        else d32[0] = d[0];
      }
    }
    // the needed players' bits
    for (int i = tid; i < R * a.eb_words; i += kSThreads) {
      const int row = i / a.eb_words, j = i - row * a.eb_words;
      if (g * R + row < a.rows) a.ebits_out[(g * R + row) * a.eb_stride + j] = nb_all[i];
    }
    __syncthreads();
  }
}

// ---------------- shared first transform P = X_c W_1 on the matrix cores ----------------

// One wave per 32x32 tile of C = A[M x K] * B[K x Nn] (row-major, fp32 in memory).
// MFMA 32x32x2 f32: lane l supplies A[row l%32][k l/32] and B[k l/32][col l%32]; the
// accumulator register i of lane l is C[8*(i/4) + 4*(l/32) + i%4][l%32].
// BF16: 32x32x8 bf16, lane l supplies k = 4*(l/32) .. +3.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void first_transform_kernel(const float* A, const float* B, float* C, int M, int K, int Nn) {
  const int lane = threadIdx.x & 63;
  const int wave_global = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int tiles_n = (Nn + 31) / 32;
  const int tiles_m = (M + 31) / 32;
  if (wave_global >= tiles_m * tiles_n) return;
  const int m0 = (wave_global / tiles_n) * 32, n0 = (wave_global % tiles_n) * 32;
  const int r = lane & 31, half = lane >> 5;
  float16_t acc;
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  const int am = m0 + r, bn = n0 + r;
  if (BF16) {
    for (int k0 = 0; k0 < K; k0 += 8) {
      short4_t av, bv;
      for (int j = 0; j < 4; ++j) {
        const int kk = k0 + 4 * half + j;
        const float x = (am < M && kk < K) ? A[(size_t)am * K + kk] : 0.f;
        const float w = (bn < Nn && kk < K) ? B[(size_t)kk * Nn + bn] : 0.f;
        av[j] = bf16_bits(x);
        bv[j] = bf16_bits(w);
      }
      acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(av, bv, acc, 0, 0, 0);
    }
  } else {
    for (int k0 = 0; k0 < K; k0 += 2) {
      const int kk = k0 + half;
      const float x = (am < M && kk < K) ? A[(size_t)am * K + kk] : 0.f;
      const float w = (bn < Nn && kk < K) ? B[(size_t)kk * Nn + bn] : 0.f;
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x, w, acc, 0, 0, 0);
    }
  }
  for (int i = 0; i < 16; ++i) {
    const int row = m0 + 8 * (i / 4) + 4 * half + (i % 4);
    if (row < M && bn < Nn) C[(size_t)row * Nn + bn] = acc[i];
  }
}

// first maximum of logits[0..C) (ties -> lowest index), one wave
__global__ void argmax_kernel(const float* logits, int C, int32_t* out) {
  const int lane = threadIdx.x;
  float best = -INFINITY;
  int arg = 0x7fffffff;
  for (int c = lane; c < C; c += 64) {
    const float v = logits[c];
    if (v > best) { best = v; arg = c; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, 64);
    const int oa = __shfl_xor(arg, o, 64);
    if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
  }
  if (lane == 0) *out = arg == 0x7fffffff ? 0 : arg;
}

__global__ void store_i32_kernel(int32_t* p, int32_t v) { *p = v; }

__global__ void fill_full_mask(uint64_t* z, int64_t W, int n) {
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= W) return;
  const uint64_t tail = (n & 63) ? ((1ull << (n & 63)) - 1ull) : ~0ull;
  z[w] = (w == W - 1) ? tail : ~0ull;
}

constexpr size_t kLdsLimit = 160 * 1024 - 512;

struct EvalLayout {
  bool rs_lds, buf_lds;
  size_t lds_bytes;
  int64_t gws_floats;  // per workgroup
  int32_t bufA, bufB;
};

void fill_rows(const ds_ctx* ctx, const ds_cgraph* cg, int32_t rows_out[DS_MAX_LAYERS + 1]) {
  const int L = ctx->L, hops = cg->info.hops;
  rows_out[0] = 0;
  for (int l = 1; l <= L; ++l) {
    int h = L - l;
    if (h > hops) h = hops;
    rows_out[l] = (int32_t)cg->info.ball[h];
  }
}

EvalLayout make_layout(const ds_ctx* ctx, const ds_cgraph* cg) {
  int32_t rows_out[DS_MAX_LAYERS + 1];
  fill_rows(ctx, cg, rows_out);
  const int L = ctx->L;
  int64_t A = ctx->dims[L], B = 1;
  for (int l = 1; l <= L; ++l) {
    const int64_t out = (int64_t)rows_out[l] * ctx->dims[l];
    if (out > A) A = out;
    if (l >= 2) {
      const int64_t q = (int64_t)rows_out[l] * ctx->dims[l - 1];
      if (q > B) B = q;
    }
  }
  EvalLayout lay;
  lay.bufA = (int32_t)A;
  lay.bufB = (int32_t)B;
  const size_t rs_b = (size_t)cg->info.num_nodes * 4, buf_b = (size_t)(A + B) * 4, fix = 64 + kWaves * 256 * 4;
  if (fix + rs_b + buf_b <= kLdsLimit) { lay.rs_lds = true; lay.buf_lds = true; }
  else if (fix + buf_b <= kLdsLimit && buf_b <= rs_b) { lay.rs_lds = false; lay.buf_lds = true; }
  else if (fix + rs_b <= kLdsLimit) { lay.rs_lds = true; lay.buf_lds = false; }
  else if (fix + buf_b <= kLdsLimit) { lay.rs_lds = false; lay.buf_lds = true; }
  else { lay.rs_lds = false; lay.buf_lds = false; }
  lay.lds_bytes = fix + (lay.rs_lds ? rs_b : 0) + (lay.buf_lds ? buf_b : 0);
  lay.gws_floats = (lay.rs_lds ? 0 : cg->info.num_nodes) + (lay.buf_lds ? 0 : (A + B));
  lay.gws_floats = (lay.gws_floats + 63) & ~(int64_t)63;
  return lay;
}

int grid_for(const ds_ctx* ctx, const EvalLayout& lay, int64_t k) {
  int occ = (int)(kLdsLimit / (lay.lds_bytes ? lay.lds_bytes : 1));
  if (occ < 1) occ = 1;
  if (occ > 2048 / kThreads) occ = 2048 / kThreads;  // resident threads per CU
  int64_t g = (int64_t)ctx->num_cus * occ;
  if (g > k) g = k;
  if (g < 1) g = 1;
  return (int)g;
}

int launch_eval(ds_ctx* ctx, const EvalArgs& a, const EvalLayout& lay, int grid) {
  const void* fn;
  if (lay.rs_lds && lay.buf_lds) fn = (const void*)masked_gcn_eval_kernel<true, true>;
  else if (lay.rs_lds) fn = (const void*)masked_gcn_eval_kernel<true, false>;
  else if (lay.buf_lds) fn = (const void*)masked_gcn_eval_kernel<false, true>;
  else fn = (const void*)masked_gcn_eval_kernel<false, false>;
  if (lay.lds_bytes > 48 * 1024)
    DS_HIP(ctx, hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lay.lds_bytes));
  if (lay.rs_lds && lay.buf_lds)
    hipLaunchKernelGGL((masked_gcn_eval_kernel<true, true>), dim3(grid), dim3(kThreads), lay.lds_bytes, ctx->stream, a);
  else if (lay.rs_lds)
    hipLaunchKernelGGL((masked_gcn_eval_kernel<true, false>), dim3(grid), dim3(kThreads), lay.lds_bytes, ctx->stream, a);
  else if (lay.buf_lds)
    hipLaunchKernelGGL((masked_gcn_eval_kernel<false, true>), dim3(grid), dim3(kThreads), lay.lds_bytes, ctx->stream, a);
  else
    hipLaunchKernelGGL((masked_gcn_eval_kernel<false, false>), dim3(grid), dim3(kThreads), lay.lds_bytes, ctx->stream, a);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

void fill_args(const ds_ctx* ctx, const ds_cgraph* cg, const EvalLayout& lay, EvalArgs* a) {
  memset(a, 0, sizeof(*a));
  a->V = (int32_t)cg->info.num_nodes;
  a->n = (int32_t)cg->info.num_players;
  a->L = ctx->L;
  a->directed = cg->info.directed;
  a->bf16 = ctx->transform_dtype == DS_BF16_IN_F32_ACC;
  for (int i = 0; i <= ctx->L; ++i) a->dims[i] = ctx->dims[i];
  fill_rows(ctx, cg, a->rows_out);
  a->W = (cg->info.num_players + 63) / 64;
  a->row_ptr = cg->row_ptr;
  a->col = cg->col;
  a->eid = cg->eid;
  a->pl = cg->pl;
  a->P = cg->P;
  for (int l = 0; l < ctx->L; ++l) {
    a->Wl[l] = ctx->W[l];
    a->bias[l] = ctx->bias[l];
  }
  a->bufA_floats = lay.bufA;
  a->bufB_floats = lay.bufB;
  a->gws_stride = lay.gws_floats;
}


struct BatchedLayout {
  bool use, deg_lds, csr_lds, ext;
  int csr_off, zs_words, eb_words;
  int grid;
  size_t lds_bytes;
  int64_t rs_floats, a_floats, b_floats, q_floats, stride;
  // external-input mode: the streaming kernel's launch and its outputs
  int64_t records, deg_blocks, eb_stride;
  int32_t E_need, stream_grid, stream_lr, cnt_words, slots;
  size_t stream_lds;
};

constexpr int64_t kPartFloats = 0;

void batched_buffers(const ds_ctx* ctx, const ds_cgraph* cg, BatchedLayout* bl) {
  int32_t rows_out[DS_MAX_LAYERS + 1];
  fill_rows(ctx, cg, rows_out);
  const int L = ctx->L;
  int64_t A = 0, B = 0, dq = 0;
  for (int l = 1; l <= L; ++l) {
    const int64_t out = (int64_t)rows_out[l] * ctx->dims[l];
    if (l & 1) { if (out > A) A = out; } else { if (out > B) B = out; }
    if (l >= 2 && (int64_t)rows_out[l] * ctx->dims[l - 1] > dq) dq = (int64_t)rows_out[l] * ctx->dims[l - 1];
  }
  bl->a_floats = A * 64;
  bl->b_floats = (B > 0 ? B : 1) * 64;
  bl->q_floats = (dq > 0 ? dq : 1) * 64;
}

// the one-coalition-per-lane kernel applies to short mask rows and enough coalitions to fill lanes
BatchedLayout make_batched_layout(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k) {
  BatchedLayout bl;
  memset(&bl, 0, sizeof(bl));
  const int64_t n = cg->info.num_players;
  const int64_t Wn = (n + 63) / 64;
  bl.use = n >= 1 && Wn <= kBWMax && k >= 256;
  if (!bl.use) return bl;
  bl.zs_words = (int)(Wn > kBW ? Wn : kBW);
  batched_buffers(ctx, cg, &bl);
  const size_t fixed = (size_t)bl.zs_words * 64 * 8 + (size_t)kWBufFloats * 4;
  bl.deg_lds = cg->info.num_nodes <= kDegLdsMaxNodes && fixed + (size_t)cg->info.num_nodes * 64 * 2 + 16 <= kLdsLimit;
  bl.rs_floats = bl.deg_lds ? 0 : cg->info.num_nodes * 64;
  bl.lds_bytes = fixed + (bl.deg_lds ? (size_t)cg->info.num_nodes * 64 * 2 : 0);
  bl.lds_bytes = (bl.lds_bytes + 15) & ~(size_t)15;
  if (bl.lds_bytes > kLdsLimit) {  // wide masks and no room left: the other kernels take over
    bl.use = false;
    return bl;
  }
  const size_t csr_bytes = 4 * (((size_t)cg->info.num_nodes + 4) & ~(size_t)3) + 8 * (((size_t)cg->info.num_entries + 3) & ~(size_t)3);
  bl.csr_lds = bl.lds_bytes + csr_bytes <= kLdsLimit;
  bl.csr_off = (int)bl.lds_bytes;
  if (bl.csr_lds) bl.lds_bytes += csr_bytes;
  bl.stride = bl.rs_floats + bl.a_floats + bl.b_floats + bl.q_floats + kPartFloats;
  const int64_t blocks = (k + 63) / 64;
  int64_t g = (int64_t)ctx->num_cus * 2;
  bl.grid = (int)(blocks < g ? blocks : g);
  return bl;
}

// Long mask rows: the streaming kernel reduces every row (or complementary pair) to degrees and entry bits, and the
// one-coalition-per-lane kernel runs the layers from those. Needs 16-bit degrees and local ids and the entry bits
// of 64 coalitions in LDS.
BatchedLayout make_stream_layout(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k, int paired) {
  BatchedLayout bl;
  memset(&bl, 0, sizeof(bl));
  const int64_t n = cg->info.num_players, V = cg->info.num_nodes;
  if (n < 1 || n > (1 << 28) || k < 256 || V > 65000 || ctx->L < 1) return bl;
  if (paired && (k & 1)) return bl;
  int h = ctx->L - 1;
  if (h > cg->info.hops) h = cg->info.hops;
  const int64_t E_need = cg->ball_entries[h];
  if (E_need > (1 << 20)) return bl;
  bl.E_need = (int32_t)E_need;
  bl.eb_words = (int)((E_need + 63) / 64 * 2);  // whole 64-entry groups (one ballot each)
  if (bl.eb_words < 2) bl.eb_words = 2;
  bl.zs_words = paired ? (bl.eb_words + 3) / 4 : bl.eb_words / 2;   // (pairs: the stored members' words only)
  bl.lds_bytes = (size_t)bl.zs_words * 64 * 8 + (size_t)kWBufFloats * 4;
  if (bl.lds_bytes > kLdsLimit) return bl;
  // the streaming kernel: R = 8 rows per workgroup if their packed 16-bit counters fit LDS, else 4 or 2
  bl.stream_lr = 3;
  const size_t stream_fixed = 32 + (size_t)kSWaves * kQueueCap * 4 + 64;
  const size_t stream_row = (size_t)((V + 3) & ~(int64_t)3) * 2 + (size_t)bl.eb_words * 4;  // 16-bit counters, needed bits
  while (bl.stream_lr > 1 && (stream_row << bl.stream_lr) + stream_fixed > kLdsLimit) --bl.stream_lr;
  bl.stream_lds = (stream_row << bl.stream_lr) + stream_fixed;
  if (bl.stream_lds > kLdsLimit) return bl;
  bl.cnt_words = (int32_t)((((V + 3) & ~(int64_t)3) << bl.stream_lr) / 2);
  bl.use = true;
  bl.ext = true;
  batched_buffers(ctx, cg, &bl);
  bl.rs_floats = 0;
  bl.stride = bl.a_floats + bl.b_floats + bl.q_floats;
  const int64_t blocks = (k + 63) / 64;
  int64_t g = (int64_t)ctx->num_cus * 4;
  bl.grid = (int)(blocks < g ? blocks : g);
  bl.records = paired ? k / 2 : k;
  bl.slots = paired ? 32 : 64;
  bl.deg_blocks = (bl.records + bl.slots - 1) / bl.slots;
  bl.eb_stride = bl.eb_words;
  int occ = (int)(kLdsLimit / bl.stream_lds);
  if (occ > 2048 / kSThreads) occ = 2048 / kSThreads;
  if (occ < 1) occ = 1;
  const int64_t groups = (bl.records + (1 << bl.stream_lr) - 1) >> bl.stream_lr;
  int64_t sg = (int64_t)ctx->num_cus * occ;
  bl.stream_grid = (int)(groups < sg ? groups : sg);
  return bl;
}

size_t stream_bytes(const BatchedLayout& bl, const ds_cgraph* cg) {
  const size_t Wn = (size_t)(cg->info.num_players + 63) / 64;
  return ds_align((size_t)cg->info.num_players * 4) + ds_align((size_t)cg->info.num_nodes * 4) * 2 + ds_align((size_t)bl.records * 4) +
         2 * (ds_align(Wn * 8) + ds_align(Wn * 4)) + ds_align(16) + ds_align((size_t)bl.E_need * 4 + 4) + ds_scan_arena_bytes((int64_t)Wn) +
         ds_align((size_t)bl.deg_blocks * cg->info.num_nodes * bl.slots * 2) + ds_align((size_t)bl.records * bl.eb_stride * 4);
}

template <bool EXT>
int launch_batched(ds_ctx* ctx, const BatchedLayout& bl, const BatchedArgs& b, int grid) {
  void (*kern)(BatchedArgs);
  if (EXT) {  // (external inputs: neither the degrees nor the local CSR are kept in LDS)
    kern = b.ext_paired ? masked_gcn_eval_batched_kernel<false, false, EXT, EXT> : masked_gcn_eval_batched_kernel<false, false, EXT, false>;
  } else if (bl.deg_lds && bl.csr_lds) kern = masked_gcn_eval_batched_kernel<true, true, false>;
  else if (bl.deg_lds) kern = masked_gcn_eval_batched_kernel<true, false, false>;
  else if (bl.csr_lds) kern = masked_gcn_eval_batched_kernel<false, true, false>;
  else kern = masked_gcn_eval_batched_kernel<false, false, false>;
  if (EXT && (bl.deg_lds || bl.csr_lds)) return ds_fail(ctx, DS_EINTERNAL, "eval: external inputs with on-chip degrees or CSR");
  if (bl.lds_bytes > 48 * 1024)
    DS_HIP(ctx, hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bl.lds_bytes));
  hipLaunchKernelGGL(kern, dim3(grid), dim3(EXT && b.ext_paired ? batched_threads<true, true>() : batched_threads<EXT>()), bl.lds_bytes,
                     ctx->stream, b);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}
}  // namespace

// ---------------- scratch memory for the entry point that may not allocate ----------------
// A file-scope device array: every GPU the library runs on holds its own copy at its own address until the
// process ends. In host code the array's name is only a stand-in for the symbol; the address on a device is
// looked up once per device (below) and that pointer is what kernels, and the workspace logic, receive.
static __device__ __align__(256) unsigned char scratch[DS_EVAL_NOALLOC_SCRATCH_BYTES];
static void* g_scratch_ptr[DS_MAX_DEVICES] = {nullptr};

int ds_static_scratch_init(int device) {
  if (device < 0 || device >= DS_MAX_DEVICES) return DS_EINVAL;
  if (g_scratch_ptr[device]) return DS_OK;
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {  // `device` is current (ds_create set it)
    (void)hipGetLastError();
    return DS_EDEVICE;
  }
  g_scratch_ptr[device] = ptr;
  return DS_OK;
}

void* ds_static_scratch(int device) { return device >= 0 && device < DS_MAX_DEVICES ? g_scratch_ptr[device] : nullptr; }

int ds_launch_first_transform(ds_ctx* ctx, const float* A, const float* B, float* C, int M, int K, int Nn, int bf16) {
  const int tiles = ((M + 31) / 32) * ((Nn + 31) / 32);
  const int blocks = (tiles + kWaves - 1) / kWaves;
  if (bf16)
    hipLaunchKernelGGL((first_transform_kernel<true>), dim3(blocks), dim3(kThreads), 0, ctx->stream, A, B, C, M, K, Nn);
  else
    hipLaunchKernelGGL((first_transform_kernel<false>), dim3(blocks), dim3(kThreads), 0, ctx->stream, A, B, C, M, K, Nn);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

int ds_launch_full_mask(ds_ctx* ctx, uint64_t* z, int64_t W, int64_t n) {
  if (W <= 0) return DS_OK;
  hipLaunchKernelGGL(fill_full_mask, dim3((unsigned)((W + 255) / 256)), dim3(256), 0, ctx->stream, z, W, (int)n);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

int ds_launch_argmax(ds_ctx* ctx, const float* logits, int C, int32_t* out) {
  hipLaunchKernelGGL(argmax_kernel, dim3(1), dim3(64), 0, ctx->stream, logits, C, out);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

// whether the single evaluation that finds the predicted class goes through the layer-by-layer kernels
static bool prepare_uses_blocks(const ds_ctx* ctx, const ds_cgraph* cg) {
  return cg->info.num_entries >= 32768 && ds_eval_zt_applies(ctx, cg, 1, 1) &&
         ds_eval_zt_arena_bytes(ctx, cg, 1, 1) <= ((size_t)1 << 30);
}

size_t ds_eval_arena_bytes(ds_ctx* ctx, const ds_cgraph* cg, int64_t k) {
  if (ctx->model_kind == DS_MODEL_GAT) return ds_gat_eval_arena_bytes(ctx, cg, k);
  const EvalLayout lay = make_layout(ctx, cg);
  const int grid = grid_for(ctx, lay, k > 1 ? k : 1);
  const size_t W = (cg->info.num_players + 63) / 64;
  const int path = ctx->tuning.eval_path;
  BatchedLayout bl;
  memset(&bl, 0, sizeof(bl));
  if (path == 0 || path == 2) bl = make_batched_layout(ctx, cg, k);
  size_t batched = bl.use ? ds_align((size_t)bl.stride * 4 * bl.grid) : 0;
  if (!bl.use && (path == 0 || path == 3)) {
    bl = make_stream_layout(ctx, cg, k, 0);  // the unpaired form is the larger one
    if (bl.use) batched = ds_align((size_t)bl.stride * 4 * bl.grid) + stream_bytes(bl, cg);
  }
  if (!bl.use && (path == 0 || path == 4)) batched = ds_eval_zt_arena_bytes(ctx, cg, k);
  // the last terms: what ds_prepare_model allocates (full mask row, logits, one workgroup's scratch or the operands
  // of one block of the layer-by-layer kernels)
  return ds_align((size_t)lay.gws_floats * 4 * grid) + batched + ds_align(W * 8 + 8) + ds_align(ctx->dims[ctx->L] * 4 + 8) +
         ds_align((size_t)lay.gws_floats * 4) + (prepare_uses_blocks(ctx, cg) ? ds_eval_zt_arena_bytes(ctx, cg, 1, 1) : 0) + 1024;
}

bool ds_eval_streams_pairs(ds_ctx* ctx, const ds_cgraph* cg, int64_t k) {
  if (ctx->model_kind == DS_MODEL_GAT || (k & 1)) return false;
  const int path = ctx->tuning.eval_path;
  if (path == 0 || path == 2) {
    if (make_batched_layout(ctx, cg, k).use) return false;
  }
  if (path == 0 || path == 3) return make_stream_layout(ctx, cg, k, 1).use;
  return false;
}

// Shared first transform and the class predicted on the full computational graph;
// cached in the graph until the model changes. Uses the arena (caller reserved it).
int ds_prepare_model(ds_ctx* ctx, ds_cgraph* cg) {
  if (ctx->L < 1) return ds_fail(ctx, DS_EINVAL, "no model is set (ds_set_gcn / ds_set_gat)");
  if (ctx->model_kind == DS_MODEL_GAT) return ds_gat_prepare_model(ctx, cg);
  if (cg->d0 != ctx->dims[0]) return ds_fail(ctx, DS_EINVAL, "feature width %d does not match the model's input width %d", cg->d0, ctx->dims[0]);
  if (cg->model_version == ctx->model_version) return DS_OK;
  if (cg->d1 != ctx->dims[1]) return ds_fail(ctx, DS_EINVAL, "the computational graph was extracted for a model with first hidden width %d (now %d): extract again", cg->d1, ctx->dims[1]);
  // The shared product is formed once per target and feeds every coalition: it stays in fp32 also in the
  // reduced-precision configuration (only the per-coalition transforms round their operands to bfloat16).
  DS_TRY(ds_launch_first_transform(ctx, cg->Xc, ctx->W[0], cg->P, (int)cg->info.num_nodes, ctx->dims[0], ctx->dims[1], 0));
  // predicted class: evaluate the full coalition once and take the first maximum
  const int64_t n = cg->info.num_players;
  const int64_t W = (n + 63) / 64;
  const int C = ctx->dims[ctx->L];
  const EvalLayout lay = make_layout(ctx, cg);
  uint64_t* zfull = (uint64_t*)ds_arena_alloc(ctx, W * 8 + 8);
  float* logits = (float*)ds_arena_alloc(ctx, C * 4 + 8);
  float* gws = lay.gws_floats ? (float*)ds_arena_alloc(ctx, (size_t)lay.gws_floats * 4) : nullptr;
  if (!zfull || !logits || (lay.gws_floats && !gws)) return ds_fail(ctx, DS_EINTERNAL, "prepare: arena exhausted");
  if (W > 0) hipLaunchKernelGGL(fill_full_mask, dim3((unsigned)((W + 255) / 256)), dim3(256), 0, ctx->stream, zfull, W, (int)n);
  EvalArgs a;
  fill_args(ctx, cg, lay, &a);
  a.Z = zfull;
  a.k = 1;
  a.y = logits + C;  // one float of scratch after the logits
  a.logits_out = logits;
  a.gws = gws;
  a.score = DS_SCORE_LOGIT;
  hipLaunchKernelGGL(store_i32_kernel, dim3(1), dim3(1), 0, ctx->stream, cg->d_pred, 0);  // a kernel, not a memset node
  a.pred_ptr = cg->d_pred;
  // a large graph: one workgroup would walk every entry alone (21 ms for 200k entries); the layer-by-layer kernels
  // spread the rows of the one coalition over the whole GPU
  // (where the workspace has the room: the entry point that may not allocate keeps the one-workgroup form)
  if (prepare_uses_blocks(ctx, cg) && ctx->arena_bytes - ctx->arena_used >= ds_eval_zt_arena_bytes(ctx, cg, 1, 1))
    DS_TRY(ds_eval_zt(ctx, cg, zfull, 1, DS_SCORE_LOGIT, logits + C, logits, cg->d_pred));
  else
    DS_TRY(launch_eval(ctx, a, lay, 1));
  hipLaunchKernelGGL(argmax_kernel, dim3(1), dim3(64), 0, ctx->stream, logits, C, cg->d_pred);
  DS_HIP(ctx, hipGetLastError());
  cg->pred_class = -1;
  cg->model_version = ctx->model_version;
  return DS_OK;
}

// flags: DS_EVAL_BOUNDED: the workspace is bounded (it is not the context's own arena): fit the launch into it;
// DS_EVAL_PAIRED: rows 2r and 2r+1 are complementary pairs (the sampler's layout)
int ds_eval_impl(ds_ctx* ctx, ds_cgraph* cg, const uint64_t* Z, int64_t k, int score, float* y, int flags, const int32_t* sz) {
  if (ctx->model_kind == DS_MODEL_GAT) return ds_gat_eval_impl(ctx, cg, Z, k, score, y);
  DS_TRY(ds_prepare_model(ctx, cg));
  if (k <= 0) return DS_OK;
  const bool bounded = (flags & DS_EVAL_BOUNDED) != 0;
  const int paired = (flags & DS_EVAL_PAIRED) != 0 && (k & 1) == 0;
  const EvalLayout lay = make_layout(ctx, cg);
  // which kernel: short mask rows -> one coalition per lane with everything on chip; long rows -> the streaming
  // kernel + the same kernel on its compact output; otherwise (few rows, very wide graphs) one workgroup per
  // coalition. ds_tuning.eval_path forces one of them where it applies (a test hook).
  const int path = ctx->tuning.eval_path;
  BatchedLayout bl;
  memset(&bl, 0, sizeof(bl));
  if (path == 0 || path == 2) bl = make_batched_layout(ctx, cg, k);
  if (!bl.use && (path == 0 || path == 3)) bl = make_stream_layout(ctx, cg, k, paired);
  if (bl.use) {
    const int64_t n = cg->info.num_players;
    BatchedArgs b;
    memset(&b, 0, sizeof(b));
    fill_args(ctx, cg, lay, &b.e);
    DS_TRY(ds_kernel_mark(ctx, 0, 0));
    if (bl.ext) {
      const int64_t Wn = (n + 63) / 64;
      uint32_t* pab = (uint32_t*)ds_arena_alloc(ctx, (size_t)n * 4);
      uint64_t* wsplit = (uint64_t*)ds_arena_alloc(ctx, (size_t)Wn * 8);
      int32_t* wfirst = (int32_t*)ds_arena_alloc(ctx, (size_t)Wn * 4);
      uint32_t* fdeg2 = (uint32_t*)ds_arena_alloc(ctx, (size_t)cg->info.num_nodes * 4);
      uint64_t* nmask = (uint64_t*)ds_arena_alloc(ctx, (size_t)Wn * 8);
      int32_t* nbase = (int32_t*)ds_arena_alloc(ctx, (size_t)Wn * 4);
      int32_t* need_range = (int32_t*)ds_arena_alloc(ctx, 16);
      int32_t* erank = (int32_t*)ds_arena_alloc(ctx, (size_t)(bl.E_need > 0 ? bl.E_need : 1) * 4);
      int32_t* sizes = sz ? nullptr : (int32_t*)ds_arena_alloc(ctx, (size_t)bl.records * 4);
      uint16_t* deg = (uint16_t*)ds_arena_alloc(ctx, (size_t)bl.deg_blocks * cg->info.num_nodes * bl.slots * 2);
      uint32_t* ebits = (uint32_t*)ds_arena_alloc(ctx, (size_t)bl.records * bl.eb_stride * 4);
      if (!pab || !wsplit || !wfirst || !fdeg2 || !nmask || !nbase || !need_range || !erank || (!sz && !sizes) || !deg || !ebits)
        return ds_fail(ctx, bounded ? DS_ECAPACITY : DS_EINTERNAL, "eval: workspace exhausted (%lld records of %lld bytes)",
                       (long long)bl.records, (long long)(cg->info.num_nodes * 2 + bl.eb_stride * 4));
      hipLaunchKernelGGL(pack_endpoints_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, cg->pl, n, pab,
                         (unsigned long long*)wsplit, wfirst);
      hipLaunchKernelGGL(full_degree_kernel, dim3((unsigned)((cg->info.num_nodes + 255) / 256)), dim3(256), 0, ctx->stream, cg->row_ptr,
                         (int)cg->info.num_nodes, fdeg2);
      // the players whose bits layer 1 reads: their words' masks, the rank of every such player, the rank per entry
      hipLaunchKernelGGL(zero_u64_kernel, dim3((unsigned)((Wn + 255) / 256)), dim3(256), 0, ctx->stream, nmask, Wn);
      if (bl.E_need > 0)
        hipLaunchKernelGGL(need_mark_kernel, dim3((unsigned)((bl.E_need + 255) / 256)), dim3(256), 0, ctx->stream, cg->eid, bl.E_need,
                           (unsigned long long*)nmask);
      hipLaunchKernelGGL(need_count_kernel, dim3((unsigned)((Wn + 255) / 256)), dim3(256), 0, ctx->stream, nmask, Wn, nbase);
      DS_TRY(ds_scan_exclusive_i32(ctx, nbase, nbase, Wn, nullptr));
      hipLaunchKernelGGL(store_i32_kernel, dim3(1), dim3(1), 0, ctx->stream, need_range, 0x7fffffff);
      hipLaunchKernelGGL(store_i32_kernel, dim3(1), dim3(1), 0, ctx->stream, need_range + 1, 0);
      hipLaunchKernelGGL(need_range_kernel, dim3((unsigned)((Wn + 255) / 256)), dim3(256), 0, ctx->stream, nmask, Wn, need_range);
      if (bl.E_need > 0)
        hipLaunchKernelGGL(need_rank_kernel, dim3((unsigned)((bl.E_need + 255) / 256)), dim3(256), 0, ctx->stream, cg->eid, bl.E_need,
                           nmask, nbase, erank);
      StreamArgs sa;
      memset(&sa, 0, sizeof(sa));
      sa.V = (int32_t)cg->info.num_nodes;
      sa.n = (int32_t)n;
      sa.directed = cg->info.directed;
      sa.E_need = bl.E_need;
      sa.W = (n + 63) / 64;
      sa.rows = bl.records;
      sa.row_stride = paired ? 2 * sa.W : sa.W;
      sa.Z = Z;
      sa.pab = pab;
      sa.wsplit = wsplit;
      sa.wfirst = wfirst;
      sa.row_ptr = cg->row_ptr;
      sa.nmask = nmask;
      sa.nbase = nbase;
      sa.need_range = need_range;
      sa.eb_words = bl.eb_words;
      sa.deg_out = deg;
      sa.ebits_out = ebits;
      sa.lr = bl.stream_lr;
      sa.cnt_words = bl.cnt_words;
      sa.slots = bl.slots;
      sa.eb_stride = bl.eb_stride;
      if (paired && ctx->lists.entries != nullptr) {  // (set by an explanation whose sampler wrote lists for these very rows)
        sa.list = ctx->lists.entries;
        sa.list_offset = ctx->lists.offset;
      }
      DS_TRY(ds_kernel_mark(ctx, 4, 0));
      if (sz) {  // the sampler's sizes: row r of this launch is row r (or 2r) of the mask matrix
        sa.sizes = sz;
        sa.size_step = paired ? 2 : 1;
      } else {
        int64_t pg = (bl.records * 64 + kThreads - 1) / kThreads;
        if (pg > (int64_t)ctx->num_cus * 32) pg = (int64_t)ctx->num_cus * 32;
        hipLaunchKernelGGL(mask_row_sizes_kernel, dim3((unsigned)pg), dim3(kThreads), 0, ctx->stream, Z, bl.records, sa.row_stride, sa.W, sizes);
        sa.sizes = sizes;
        sa.size_step = 1;
      }
      {
        const void* fn;
        void (*kern)(StreamArgs);
        if (paired) kern = bl.stream_lr == 3 ? stream_degrees_kernel<true, 3> : bl.stream_lr == 2 ? stream_degrees_kernel<true, 2> : stream_degrees_kernel<true, 1>;
        else kern = bl.stream_lr == 3 ? stream_degrees_kernel<false, 3> : bl.stream_lr == 2 ? stream_degrees_kernel<false, 2> : stream_degrees_kernel<false, 1>;
        fn = (const void*)kern;
        if (bl.stream_lds > 48 * 1024)
          DS_HIP(ctx, hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bl.stream_lds));
        hipLaunchKernelGGL(kern, dim3(bl.stream_grid), dim3(kSThreads), bl.stream_lds, ctx->stream, sa);
      }
      DS_HIP(ctx, hipGetLastError());
      DS_TRY(ds_kernel_mark(ctx, 4, 1));
      b.ext_deg = deg;
      b.ext_lr = bl.stream_lr;
      b.ext_bits = ebits;
      b.erank = erank;
      b.fdeg2 = fdeg2;
      b.eb_stride = bl.eb_stride;
      b.ext_paired = paired;
      b.eb_words = bl.eb_words;
    }
    // a bounded workspace (the entry point that may not allocate) runs fewer workgroups at a time instead of failing
    const size_t avail = ctx->arena_bytes - ctx->arena_used > 512 ? ctx->arena_bytes - ctx->arena_used - 512 : 0;
    int bgrid = bl.grid;
    if (bounded) {
      const size_t fit = avail / ((size_t)bl.stride * 4);
      if (fit < 1) return ds_fail(ctx, DS_ECAPACITY, "eval: one workgroup needs %zu bytes of scratch, %zu are left", (size_t)bl.stride * 4, avail);
      if ((size_t)bgrid > fit) bgrid = (int)fit;
    }
    float* scratch = (float*)ds_arena_alloc(ctx, (size_t)bl.stride * 4 * bgrid);
    if (!scratch) return ds_fail(ctx, DS_EINTERNAL, "eval: arena exhausted");
    b.e.Z = Z;
    b.e.k = k;
    b.e.y = y;
    b.e.logits_out = nullptr;
    b.e.gws = nullptr;
    b.e.score = score;
    b.e.pred_ptr = cg->d_pred;
    b.scratch = scratch;
    b.scratch_stride = bl.stride;
    b.rs_floats = bl.rs_floats;
    b.a_floats = bl.a_floats;
    b.b_floats = bl.b_floats;
    b.q_floats = bl.q_floats;
    b.csr_lds_offset = bl.csr_off;
    b.zs_words = bl.zs_words;
    if (bl.ext) DS_TRY(launch_batched<true>(ctx, bl, b, bgrid));
    else DS_TRY(launch_batched<false>(ctx, bl, b, bgrid));
    return ds_kernel_mark(ctx, 0, 1);
  }
  // graphs neither of the two can take (needed entries that do not fit LDS for 64 coalitions): layer by layer over
  // blocks of 64 coalitions, from a transposed mask matrix (needs a large workspace: not for the bounded form)
  if (!bounded && (path == 0 || path == 4) && ds_eval_zt_applies(ctx, cg, k)) {
    DS_TRY(ds_kernel_mark(ctx, 0, 0));
    DS_TRY(ds_eval_zt(ctx, cg, Z, k, score, y, nullptr, cg->d_pred, paired));
    return ds_kernel_mark(ctx, 0, 1);
  }
  const size_t avail = ctx->arena_bytes - ctx->arena_used > 512 ? ctx->arena_bytes - ctx->arena_used - 512 : 0;
  int grid = grid_for(ctx, lay, k);
  float* gws = nullptr;
  if (lay.gws_floats) {
    if (bounded) {
      const size_t fit = avail / ((size_t)lay.gws_floats * 4);
      if (fit < 1) return ds_fail(ctx, DS_ECAPACITY, "eval: one workgroup needs %zu bytes of scratch, %zu are left", (size_t)lay.gws_floats * 4, avail);
      if ((size_t)grid > fit) grid = (int)fit;
    }
    gws = (float*)ds_arena_alloc(ctx, (size_t)lay.gws_floats * 4 * grid);
    if (!gws) return ds_fail(ctx, DS_EINTERNAL, "eval: arena exhausted");
  }
  EvalArgs a;
  fill_args(ctx, cg, lay, &a);
  a.Z = Z;
  a.k = k;
  a.y = y;
  a.logits_out = nullptr;
  a.gws = gws;
  a.score = score;
  a.pred_ptr = cg->d_pred;
  DS_TRY(ds_kernel_mark(ctx, 0, 0));
  DS_TRY(launch_eval(ctx, a, lay, grid));
  return ds_kernel_mark(ctx, 0, 1);
}

int ds_fetch_pred_class(ds_ctx* ctx, ds_cgraph* cg) {
  if (cg->pred_class >= 0) return DS_OK;
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail + 34, cg->d_pred, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  cg->pred_class = *(int32_t*)(ctx->h_mail + 34);
  return DS_OK;
}
