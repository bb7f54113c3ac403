// Masked GCN inference for computational graphs whose first layer reads (nearly) every player: one layer at a
// time over blocks of 64 coalitions, from a transposed mask matrix.
//
// Paper, "Distributed Model Prediction": cost O(b (n d + |V_c| d^2)) per batch of b sub-graphs; the n d term is the
// masked aggregation. When the target is a hub, the rows the first layer has to produce hold most of the graph's
// entries (a 100k-player graph: 196k of 200k CSR entries), and one workgroup per coalition pays one gathered
// feature row per active entry and coalition. Here 64 coalitions are evaluated together: with the mask matrix
// transposed block-wise, T[block][player] = the player's bits in the block's 64 coalitions, one 8-byte word says for
// all 64 coalitions whether an entry is active, every row of P = X_c W_1 is loaded once per 64 coalitions, and
//   H1[t][f][c] = sum_e P[src_e][f] * (bit_e(c) ? d_src(c)^-1/2 : 0)
// is an (entries x coalitions)^T . (entries x features) product on the matrix cores (v_mfma_f32_32x32x2f32). Unlike the
// one-coalition-per-lane kernel for short mask rows, nothing here has to fit a workgroup's LDS: every stage is a
// kernel of its own, a bounded number of blocks at a time, with the per-coalition layer outputs [coalition][row][feature]
// in global memory (a layer that another one follows is stored times d^-1/2 of its own row, the only form the next
// aggregation uses it in):
//   degrees  d(v) = 1 + sum of the bits of row v's entries            (one wave per (block, node), lane = coalition)
//   layer 1  the contraction above, scaled by d_t^-1/2, + bias, ReLU   (one wave per (block, row), matrix cores)
//   layer l >= 2: q = D^-1/2 (A_S + I) D^-1/2 H  (one wave per (coalition, row), lanes = features, only the coalition's
//                 active entries are visited), then act(q W_l + b_l) as a (rows x features) product per coalition,
//                 matrix cores
//   readout  soft-max (or logit) of the predicted class.
// With complementary pairs only the stored members are transposed: a block is 64 stored members or their 64 complements
// (the same words inverted), and a block of sparse members skips the entries none of its coalitions has.
#include "internal.h"
#include "solve_common.h"

namespace {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef short short4_t __attribute__((ext_vector_type(4)));

constexpr int kZThreads = 256;
constexpr int kZWaves = kZThreads / 64;

struct ZtArgs {
  int32_t V, L, score, bf16;
  int32_t paired;      // rows 2r, 2r+1 are complementary: T holds the even rows only, block 2j = the stored members of pairs
                       // 64j .. 64j+63, block 2j+1 = their complements (the same words inverted)
  int32_t dims[DS_MAX_LAYERS + 1];
  int32_t rows_out[DS_MAX_LAYERS + 1];
  const int32_t *row_ptr, *col, *eid;
  const float* P;
  const float* Wl[DS_MAX_LAYERS];
  const float* bias[DS_MAX_LAYERS];
  const uint64_t* T;   // [blocks][npad]
  int64_t npad, k;
  int64_t blk0;        // first block of this launch
  int32_t nblk;        // blocks of this launch
  float* rs;           // [nblk][V][64]: d^-1/2
  const int32_t* pred_ptr;
  float* y;
  float* logits_out;   // optional: [k x d_L]
};

__device__ __forceinline__ float zt_bf16_round(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest even (finite inputs)
  return __uint_as_float(u & 0xFFFF0000u);
}

__device__ __forceinline__ uint32_t rl(uint32_t v, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)v, l); }

// the transposed words of block blk: T row and the mask to XOR onto every word (all ones for a block of complements)
__device__ __forceinline__ const uint64_t* block_words(const ZtArgs& a, int64_t blk, uint64_t* inv) {
  if (a.paired) {
    *inv = (blk & 1) ? ~0ull : 0ull;
    return a.T + (blk >> 1) * a.npad;
  }
  *inv = 0ull;
  return a.T + blk * a.npad;
}
// mask row of lane `lane` of block blk
__device__ __forceinline__ int64_t block_row(const ZtArgs& a, int64_t blk, int lane) {
  return a.paired ? 2 * ((blk >> 1) * 64 + lane) + (blk & 1) : blk * 64 + lane;
}

// d(v)^-1/2 for every node and coalition of the launch's blocks. One wave per (block, node): the lanes fetch the
// words of up to 64 entries of the row together, then every word is broadcast and each lane adds its own bit.
__global__ __launch_bounds__(kZThreads) void zt_degrees_kernel(ZtArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * kZThreads + threadIdx.x) >> 6, nwaves = ((int64_t)gridDim.x * kZThreads) >> 6;
  const uint32_t mlo = lane < 32 ? 1u << lane : 0u, mhi = lane >= 32 ? 1u << (lane - 32) : 0u;
  const int64_t tasks = (int64_t)a.nblk * a.V;
  for (int64_t task = wave; task < tasks; task += nwaves) {
    const int64_t cbi = task / a.V;
    const int v = (int)(task - cbi * a.V);
    uint64_t inv;
    const uint64_t* Tb = block_words(a, a.blk0 + cbi, &inv);
    const int e0 = a.row_ptr[v], e1 = a.row_ptr[v + 1];
    int cnt = 1;
    for (int eb = e0; eb < e1; eb += 64) {
      const int m = e1 - eb < 64 ? e1 - eb : 64;
      const uint64_t word = lane < m ? Tb[a.eid[eb + lane]] ^ inv : 0ull;
      const uint32_t lo = (uint32_t)word, hi = (uint32_t)(word >> 32);
      for (int i = 0; i < m; ++i) cnt += ((rl(lo, i) & mlo) | (rl(hi, i) & mhi)) ? 1 : 0;
    }
    a.rs[((size_t)cbi * a.V + v) * 64 + lane] = 1.0f / sqrtf((float)cnt);
  }
}

// Layer 1 on the matrix cores, one wave per (block, row t): H1[t][f][c] = act( d_t(c)^-1/2 sum_e P[src_e][f] coef_e(c)
// + b[f] ), the sum over the row's entries and the self-loop (coef = d_t^-1/2). With v_mfma_f32_32x32x2f32 lane l
// supplies A[m = l%32][k = l/32] = P[src of entry 2q + l/32][f0 + l%32] and B[k = l/32][n = l%32] = coefficient of
// entry 2q + l/32 for coalition n (and, for the second accumulator column, coalition 32 + n): a lane reads the
// degree factors of exactly the two coalitions it feeds and tests their two bits of the entry's word, so no
// value crosses lanes. Entries are fetched 64 at a time (lane j: entry j's source, word), steps of two entries; the
// operands of four steps are requested together. Rows are short (20 entries on the hub workload), so a task is mostly
// the chain row bounds -> entries -> words -> operands: four workgroups a compute unit (the accumulators in ordinary
// registers, 117 in all) hide it better than two (29 -> 19 ms there).
__global__ __launch_bounds__(kZThreads, 4) void zt_layer1_kernel(ZtArgs a, float* out) {
  const int lane = threadIdx.x & 63, half = lane >> 5, l32 = lane & 31;
  const int64_t wave = ((int64_t)blockIdx.x * kZThreads + threadIdx.x) >> 6, nwaves = ((int64_t)gridDim.x * kZThreads) >> 6;
  const int d1 = a.dims[1], rows1 = a.rows_out[1];
  const bool relu = a.L > 1;
  const int64_t tasks = (int64_t)a.nblk * rows1;
  for (int64_t task = wave; task < tasks; task += nwaves) {
    const int64_t cbi = task / rows1;
    const int t = (int)(task - cbi * rows1);
    uint64_t inv;
    const uint64_t* Tb = block_words(a, a.blk0 + cbi, &inv);
    const float* rsb = a.rs + (size_t)cbi * a.V * 64;
    const int e0 = a.row_ptr[t], e1 = a.row_ptr[t + 1];  // entry e1 stands for the self-loop
    const float rst0 = rsb[(size_t)t * 64 + l32], rst1 = rsb[(size_t)t * 64 + 32 + l32];
    for (int f0 = 0; f0 < d1; f0 += 64) {
      float16_t acc[2][2];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        acc[0][0][i] = 0.f; acc[0][1][i] = 0.f; acc[1][0][i] = 0.f; acc[1][1][i] = 0.f;
      }
      const bool fok0 = f0 + l32 < d1, fok1 = f0 + 32 + l32 < d1;
      for (int eb = e0; eb <= e1; eb += 64) {
        const int m = e1 + 1 - eb < 64 ? e1 + 1 - eb : 64;
        const int e = eb + lane;
        int sv = t;
        uint64_t word = 0ull;
        if (e < e1) {
          sv = a.col[e];
          word = Tb[a.eid[e]] ^ inv;
        } else if (e == e1) {
          word = ~0ull;
        }
        const uint32_t wlo = (uint32_t)word, whi = (uint32_t)(word >> 32);
        // only entries that are active in some coalition of the block take a step (in a block of sparse stored members
        // most are not): their lanes are taken from the ballot, eight at a time = four steps of two entries
        unsigned long long act = __ballot(word != 0ull);
        while (act) {
          int il[8];
          bool live[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            live[j] = act != 0ull;
            il[j] = live[j] ? __ffsll((long long)act) - 1 : 63;
            act &= act - 1ull;
          }
          float av[4][2], rv[4][2];
          uint32_t b0m[4], b1m[4];
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            const int il0 = il[2 * s], il1 = il[2 * s + 1];
            const int s0 = (int)rl((uint32_t)sv, il0), s1 = (int)rl((uint32_t)sv, il1);
            const uint32_t l0 = rl(wlo, il0), l1 = rl(wlo, il1), h0 = rl(whi, il0), h1 = rl(whi, il1);
            const bool live0 = live[2 * s], live1 = live[2 * s + 1];
            const int src = half ? s1 : s0;
            const uint32_t lo = half ? (live1 ? l1 : 0u) : (live0 ? l0 : 0u);
            const uint32_t hi = half ? (live1 ? h1 : 0u) : (live0 ? h0 : 0u);
            b0m[s] = (lo >> l32) & 1u;
            b1m[s] = (hi >> l32) & 1u;
            // (loads issued unconditionally, a feature past the end reads column 0 and is zeroed: a wait for operands
            // is then a count of younger loads)
            const float* pr = a.P + (size_t)src * d1;
            const float x0 = pr[fok0 ? f0 + l32 : 0], x1 = pr[fok1 ? f0 + 32 + l32 : 0];
            av[s][0] = fok0 ? x0 : 0.f;
            av[s][1] = fok1 ? x1 : 0.f;
            const float* rp = rsb + (size_t)src * 64 + l32;
            rv[s][0] = rp[0];
            rv[s][1] = rp[32];
          }
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            if (live[2 * s]) {
              const float b0 = b0m[s] ? rv[s][0] : 0.f, b1 = b1m[s] ? rv[s][1] : 0.f;
              // (coefficients as the A operand, rows of P as B: the accumulator is [coalition][feature])
              acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(b0, av[s][0], acc[0][0], 0, 0, 0);
              acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(b1, av[s][0], acc[0][1], 0, 0, 0);
              acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(b0, av[s][1], acc[1][0], 0, 0, 0);
              acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(b1, av[s][1], acc[1][1], 0, 0, 0);
            }
          }
        }
      }
      // accumulator register i of lane l of acc[ft][nb] is D[coalition 32*nb + 8*(i/4) + 4*(l/32) + i%4][feature f0 + 32*ft +
      // l%32]: a store is 128 contiguous bytes of one coalition's row. A layer that another one follows is stored
      // already multiplied by d_t^-1/2 (the only form the next aggregation uses it in).
      // (the four coalitions of a register group are consecutive: their d_t^-1/2 come as one 16-byte load, and the
      // store address advances by one coalition's array at a time instead of being formed 64 times over)
      const size_t cs = (size_t)rows1 * d1;   // floats between two coalitions
      float* o = out + (((size_t)cbi * 64 + 4 * half) * rows1 + t) * d1 + f0 + l32;
      const float* rp = rsb + (size_t)t * 64 + 4 * half;
      const bool ok0 = f0 + l32 < d1, ok1 = f0 + 32 + l32 < d1;
      const float bias0 = (a.bias[0] && ok0) ? a.bias[0][f0 + l32] : 0.f, bias1 = (a.bias[0] && ok1) ? a.bias[0][f0 + 32 + l32] : 0.f;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 rt4 = *(const float4*)(rp + 32 * nb + 8 * g);
          const float rt[4] = {rt4.x, rt4.y, rt4.z, rt4.w};
          float* og = o + (size_t)(32 * nb + 8 * g) * cs;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            float v0 = rt[j] * acc[0][nb][4 * g + j] + bias0, v1 = rt[j] * acc[1][nb][4 * g + j] + bias1;
            if (relu) {
              v0 = fmaxf(v0, 0.f) * rt[j];
              v1 = fmaxf(v1, 0.f) * rt[j];
            }
            if (ok0) og[0] = v0;
            if (ok1) og[32] = v1;
            og += cs;
          }
        }
    }
  }
}

// Aggregation of a later layer, one wave per (coalition, row t), lanes = features: q[t][f] = d_t^-1/2 ( sum over the
// ACTIVE entries of H'[src][f] + H'[t][f] ), H' being the previous layer's output times d^-1/2 of its own row (stored that
// way). Only the coalition's own active entries are visited: the lanes test the bits of 64 entries together and the set
// ones are walked eight at a time (eight 256-byte row loads in flight). The layer's input of one coalition (rows x d x 4
// bytes: 2.5 MB on the hub workload) is read by all rows t of that coalition, about sixteen times over; with one row per
// wave the whole GPU works on a few dozen coalitions at a time, so those re-reads come from the caches (HBM traffic of
// the hub workload's second layer: 780 GB as [row][feature][64 coalitions] -> 53 GB). The launch also keeps the workgroups
// of a coalition on one XCD (workgroups go to the XCDs round-robin by index); measured, that made no difference
// against plain order.
__global__ __launch_bounds__(kZThreads) void zt_aggregate_kernel(ZtArgs a, int l, const float* cur, float* q, int wg_per_coalition) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int din = a.dims[l - 1], rows = a.rows_out[l], rows_prev = a.rows_out[l - 1];
  const int xcd = blockIdx.x & 7;
  const int64_t slot = blockIdx.x >> 3;
  const int64_t cl = (slot / wg_per_coalition) * 8 + xcd;   // coalition of the launch
  const int t = (int)(slot % wg_per_coalition) * kZWaves + wave;
  if (cl >= (int64_t)a.nblk * 64 || t >= rows) return;
  const int64_t cbi = cl >> 6;
  const int cb = (int)(cl & 63);   // the coalition's bit in its block's words
  if (block_row(a, a.blk0 + cbi, cb) >= a.k) return;
  uint64_t inv;
  const uint64_t* Tb = block_words(a, a.blk0 + cbi, &inv);
  const float rst = a.rs[((size_t)cbi * a.V + t) * 64 + cb];
  const float* hb = cur + (size_t)cl * rows_prev * din;
  const int e0 = a.row_ptr[t], e1 = a.row_ptr[t + 1];  // entry e1 stands for the self-loop
  for (int f0 = 0; f0 < din; f0 += 64) {
    const bool fok = f0 + lane < din;
    const float* hf = hb + (fok ? f0 + lane : 0);
    float acc = 0.f;
    for (int eb = e0; eb <= e1; eb += 64) {
      const int e = eb + lane;
      int sv = t;
      bool on = e == e1;
      if (e < e1) {
        sv = a.col[e];
        on = ((Tb[a.eid[e]] ^ inv) >> cb) & 1ull;
      }
      unsigned long long act = __ballot(on);
      while (act) {
        float hv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const bool live = act != 0ull;
          const int i = live ? __ffsll((long long)act) - 1 : 63;
          act &= act - 1ull;
          const int src = (int)rl((uint32_t)sv, i);
          const float x = hf[(size_t)src * din];   // (issued unconditionally; a spent slot reads a valid row and adds zero)
          hv[u] = live ? x : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += hv[u];
      }
    }
    if (fok) {
      const float v = rst * acc;
      q[((size_t)cl * rows + t) * din + f0 + lane] = a.bf16 ? zt_bf16_round(v) : v;
    }
  }
}

// Dense transform of a later layer on the matrix cores, per coalition: nxt[t][j] = act( sum_f q[t][f] W[f][j] + b[j] ), a
// (rows x features in) . (features in x features out) product. One wave per (coalition, 32 rows, 32 output features):
// lane l supplies q[t0 + l%32][f + l/32] (eight consecutive f of its row per load pair) and W[f + l/32][j0 + l%32]
// (v_mfma_f32_32x32x2f32); in the bfloat16 configuration both operands are rounded to bfloat16 (q already is) and
// v_mfma_f32_32x32x8bf16_1k accumulates in fp32, lane l supplying f = 4*(l/32) .. +3. A layer that another one follows
// is stored times d_t^-1/2.
__global__ __launch_bounds__(kZThreads) void zt_transform_kernel(ZtArgs a, int l, const float* q, float* nxt) {
  const int lane = threadIdx.x & 63, half = lane >> 5, r = lane & 31;
  const int64_t wave = ((int64_t)blockIdx.x * kZThreads + threadIdx.x) >> 6, nwaves = ((int64_t)gridDim.x * kZThreads) >> 6;
  const int din = a.dims[l - 1], dout = a.dims[l], rows = a.rows_out[l];
  const bool last = l == a.L, isbf = a.bf16 != 0;
  const float* Wg = a.Wl[l - 1];
  const float* bias = a.bias[l - 1];
  const int jt = (dout + 31) / 32, tt = (rows + 31) / 32;
  const int64_t tasks = (int64_t)a.nblk * 64 * tt * jt;
  for (int64_t task = wave; task < tasks; task += nwaves) {
    const int64_t cl = task / (tt * jt);
    const int rem = (int)(task - cl * tt * jt);
    const int t0 = (rem / jt) * 32, j0 = (rem % jt) * 32;
    const int64_t cbi = cl >> 6;
    const int cb = (int)(cl & 63);
    if (block_row(a, a.blk0 + cbi, cb) >= a.k) continue;
    const bool jok = j0 + r < dout;
    const int tr = t0 + r < rows ? t0 + r : rows - 1;   // rows past the end read the last one and are not stored
    const float* qp = q + ((size_t)cl * rows + tr) * din;
    const float* wp = Wg + (jok ? j0 + r : 0);
    float16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    for (int fb = 0; fb < din; fb += 8) {
      if (isbf) {
        short4_t av, bv;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int f = fb + 4 * half + u;
          const bool ok = f < din;
          const float qv = qp[ok ? f : 0], wv = wp[(size_t)(ok ? f : 0) * dout];
          av[u] = (short)(__float_as_uint(ok ? qv : 0.f) >> 16);
          bv[u] = (short)(__float_as_uint((ok && jok) ? zt_bf16_round(wv) : 0.f) >> 16);
        }
        acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(av, bv, acc, 0, 0, 0);
      } else {
        float xa[4], xb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int f = fb + 2 * u + half;
          const bool ok = f < din;
          const float qv = qp[ok ? f : 0], wv = wp[(size_t)(ok ? f : 0) * dout];
          xa[u] = ok ? qv : 0.f;
          xb[u] = (ok && jok) ? wv : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (fb + 2 * u < din) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[u], xb[u], acc, 0, 0, 0);
      }
    }
    // accumulator register i of lane l is out[row t0 + 8*(i/4) + 4*(l/32) + i%4][feature j0 + l%32]
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int t = t0 + 8 * (i / 4) + 4 * half + (i % 4);
      if (t < rows && jok) {
        float v = acc[i] + (bias ? bias[j0 + r] : 0.f);
        if (!last) v = fmaxf(v, 0.f) * a.rs[((size_t)cbi * a.V + t) * 64 + cb];
        nxt[((size_t)cl * rows + t) * dout + j0 + r] = v;
      }
    }
  }
}

// readout: the target is row 0 of the last layer's output; one thread per coalition
__global__ void zt_readout_kernel(ZtArgs a, const float* cur) {
  const int64_t cl = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (cl >= (int64_t)a.nblk * 64) return;
  const int64_t row = block_row(a, a.blk0 + (cl >> 6), (int)(cl & 63));
  if (row >= a.k) return;
  const int C = a.dims[a.L], rowsL = a.rows_out[a.L];
  const float* lg = cur + (size_t)cl * rowsL * C;
  float m = -INFINITY;
  for (int c = 0; c < C; ++c) m = fmaxf(m, lg[c]);
  float sum = 0.f;
  for (int c = 0; c < C; ++c) sum += expf(lg[c] - m);
  const float zc = lg[*a.pred_ptr];
  a.y[row] = a.score == DS_SCORE_LOGIT ? zc : expf(zc - m) / sum;
  if (a.logits_out)
    for (int c = 0; c < C; ++c) a.logits_out[row * C + c] = lg[c];
}

struct ZtPlan {
  bool use;
  int64_t blocks, tblocks, npad, chunk;   // blocks of 64 coalitions, blocks of the transposed matrix, padded players, blocks per launch
  int64_t rs_f, a_f, b_f, q_f;        // floats per block of the four scratch regions
  int32_t rows_out[DS_MAX_LAYERS + 1];
};

constexpr size_t kZtMaxTransposed = (size_t)16 << 30;  // the transposed mask matrix may take this much
constexpr size_t kZtScratch = (size_t)6 << 30;         // per-launch operands of the blocks in flight

ZtPlan zt_plan(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k, int64_t min_rows, int paired) {
  ZtPlan p;
  memset(&p, 0, sizeof(p));
  const int64_t n = cg->info.num_players, V = cg->info.num_nodes;
  const int L = ctx->L;
  if (n < 1 || k < min_rows || L < 1 || ctx->model_kind != DS_MODEL_GCN) return p;
  p.tblocks = paired ? (k / 2 + 63) / 64 : (k + 63) / 64;   // blocks of 64 transposed rows
  p.blocks = paired ? 2 * p.tblocks : p.tblocks;
  p.npad = (n + 63) / 64 * 64;
  if ((size_t)p.tblocks * p.npad * 8 > kZtMaxTransposed) return p;
  p.rows_out[0] = 0;
  for (int l = 1; l <= L; ++l) {
    int h = L - l;
    if (h > cg->info.hops) h = cg->info.hops;
    p.rows_out[l] = (int32_t)cg->info.ball[h];
  }
  p.rs_f = V * 64;
  // layer l's output lands in region A for odd l, B for even l; q holds the aggregated rows of the layer in flight
  for (int l = 1; l <= L; ++l) {
    const int64_t out = (int64_t)p.rows_out[l] * ctx->dims[l] * 64;
    if (l & 1) p.a_f = out > p.a_f ? out : p.a_f;
    else p.b_f = out > p.b_f ? out : p.b_f;
    if (l >= 2) {
      const int64_t qf = (int64_t)p.rows_out[l] * ctx->dims[l - 1] * 64;
      p.q_f = qf > p.q_f ? qf : p.q_f;
    }
  }
  const size_t per_block = (size_t)(p.rs_f + p.a_f + p.b_f + p.q_f) * 4;
  int64_t c = (int64_t)(kZtScratch / per_block);
  if (c < 1) c = 1;
  if (c > p.blocks) c = p.blocks;
  p.chunk = c;
  p.use = true;
  return p;
}

int64_t grid_for_waves(const ds_ctx* ctx, int64_t tasks) {
  int64_t g = (tasks + kZWaves - 1) / kZWaves;
  const int64_t cap = (int64_t)ctx->num_cus * 8;
  if (g > cap) g = cap;
  return g < 1 ? 1 : g;
}

}  // namespace

// (a block of 64 coalitions is the unit of work: with fewer than min_rows rows the other kernels are the better choice,
// except for the single evaluation of a large graph, where one workgroup would walk every entry alone)
bool ds_eval_zt_applies(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k, int64_t min_rows) { return zt_plan(ctx, cg, k, min_rows, 0).use; }

size_t ds_eval_zt_arena_bytes(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k, int64_t min_rows) {
  // (the paired form holds half the transposed matrix and may run one block more at a time: room for either)
  const ZtPlan p = zt_plan(ctx, cg, k, min_rows, 0);
  if (!p.use) return 0;
  const size_t c = (size_t)p.chunk + 1;
  return ds_align((size_t)p.tblocks * p.npad * 8) + ds_align((size_t)p.rs_f * 4 * c) + ds_align((size_t)p.a_f * 4 * c) +
         ds_align((size_t)p.b_f * 4 * c + 256) + ds_align((size_t)p.q_f * 4 * c + 256) + 1024;
}

// The model must be prepared (P and the predicted class on the device); temporaries come from the context's arena.
int ds_eval_zt(ds_ctx* ctx, ds_cgraph* cg, const uint64_t* Z, int64_t k, int score, float* y, float* logits_out,
               const int32_t* pred_ptr, int paired) {
  paired = paired && (k & 1) == 0 && k >= 2;
  const ZtPlan p = zt_plan(ctx, cg, k, 1, paired);
  if (!p.use) return ds_fail(ctx, DS_EINTERNAL, "eval: the block-transposed path does not apply");
  const int64_t n = cg->info.num_players, W = (n + 63) / 64;
  uint64_t* T = (uint64_t*)ds_arena_alloc(ctx, (size_t)p.tblocks * p.npad * 8);
  float* rs = (float*)ds_arena_alloc(ctx, (size_t)p.rs_f * 4 * p.chunk);
  float* bufA = (float*)ds_arena_alloc(ctx, (size_t)p.a_f * 4 * p.chunk);
  float* bufB = (float*)ds_arena_alloc(ctx, (size_t)p.b_f * 4 * p.chunk + 256);
  float* q = (float*)ds_arena_alloc(ctx, (size_t)p.q_f * 4 * p.chunk + 256);
  if (!T || !rs || !bufA || !bufB || !q) return ds_fail(ctx, DS_EINTERNAL, "eval: arena exhausted");
  // (pairs: only the stored members, rows 0, 2, 4, ...)
  DS_TRY(ds_bit_transpose_blocks(ctx, Z, paired ? k / 2 : k, n, W, paired ? 2 : 1, T));
  ZtArgs a;
  memset(&a, 0, sizeof(a));
  a.V = (int32_t)cg->info.num_nodes;
  a.L = ctx->L;
  a.score = score;
  a.bf16 = ctx->transform_dtype == DS_BF16_IN_F32_ACC;
  a.paired = paired;
  for (int i = 0; i <= ctx->L; ++i) {
    a.dims[i] = ctx->dims[i];
    a.rows_out[i] = p.rows_out[i];
  }
  a.row_ptr = cg->row_ptr;
  a.col = cg->col;
  a.eid = cg->eid;
  a.P = cg->P;
  for (int l = 0; l < ctx->L; ++l) {
    a.Wl[l] = ctx->W[l];
    a.bias[l] = ctx->bias[l];
  }
  a.T = T;
  a.npad = p.npad;
  a.k = k;
  a.rs = rs;
  a.pred_ptr = pred_ptr;
  a.y = y;
  a.logits_out = logits_out;
  for (int64_t b0 = 0; b0 < p.blocks; b0 += p.chunk) {
    a.blk0 = b0;
    a.nblk = (int32_t)(p.blocks - b0 < p.chunk ? p.blocks - b0 : p.chunk);
    hipLaunchKernelGGL(zt_degrees_kernel, dim3((unsigned)grid_for_waves(ctx, (int64_t)a.nblk * a.V)), dim3(kZThreads), 0, ctx->stream, a);
    hipLaunchKernelGGL(zt_layer1_kernel, dim3((unsigned)grid_for_waves(ctx, (int64_t)a.nblk * a.rows_out[1])), dim3(kZThreads), 0,
                       ctx->stream, a, bufA);
    float* cur = bufA;
    for (int l = 2; l <= ctx->L; ++l) {
      float* nxt = (l & 1) ? bufA : bufB;
      const int wg_per_coalition = (a.rows_out[l] + kZWaves - 1) / kZWaves;
      const int64_t agg_grid = (((int64_t)a.nblk * 64 + 7) / 8) * wg_per_coalition * 8;
      const int64_t tt = (a.rows_out[l] + 31) / 32, jt = (a.dims[l] + 31) / 32;
      if (agg_grid > 0x7fffffffLL) return ds_fail(ctx, DS_EINTERNAL, "eval: too many aggregation workgroups");
      hipLaunchKernelGGL(zt_aggregate_kernel, dim3((unsigned)agg_grid), dim3(kZThreads), 0, ctx->stream, a, l, (const float*)cur, q,
                         wg_per_coalition);
      hipLaunchKernelGGL(zt_transform_kernel, dim3((unsigned)grid_for_waves(ctx, (int64_t)a.nblk * 64 * tt * jt)), dim3(kZThreads), 0,
                         ctx->stream, a, l, (const float*)q, nxt);
      cur = nxt;
    }
    hipLaunchKernelGGL(zt_readout_kernel, dim3((unsigned)((a.nblk * 64 + 255) / 256)), dim3(256), 0, ctx->stream, a, (const float*)cur);
  }
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}
