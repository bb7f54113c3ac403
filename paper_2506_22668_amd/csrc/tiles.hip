// The sparse rows of the CGLS matrix (paper, Alg. 1: both products with the mask matrix, here the small members of the
// pairs that hold few players) as 2-D tiles of (row, column) entries, multiplied both ways through LDS.
//
// One index-list entry per set bit and one gather per entry from a vector in global memory fetches a whole cache line
// for eight bytes: that, not the index traffic, bounded the index-list products. Here the entries of a (row block x
// column chunk) tile (at most 8192 rows x 8192 columns, entry = 13 + 13 bits in a u32) are multiplied with both
// vector pieces in LDS: the source piece as 64-bit fixed point (the same scaled integers the matrix-core product of
// the dense rows uses, a few low bits dropped with rounding so that a whole accumulator fits 63 bits), the target piece
// as 64-bit LDS accumulators added to with LDS atomics. Integer addition is exact and commutative, so neither the
// order of the entries inside a tile nor the order of the atomics can change a result: the same list, in whatever order
// the build left it, serves  d = S u  (accumulate by row, gather by column) and  s = S^T h  (accumulate by column,
// gather by row), and no transposed copy is built.
//
// Row blocks hold at most 8192 rows and about 1/16 of the entries each (the rows are sorted by size, so the blocks of
// the largest rows are short; a tile of such a block holds several times more entries than the 8192 source values
// staged for it); workgroups of the forward product own (row block, group of chunks),
// those of the adjoint (chunk, group of row blocks of at most 32768 rows): both are balanced in entries. Tiles with few
// entries gather from the global copy instead of staging a source piece.
#include "internal.h"
#include "solve_common.h"

namespace {
constexpr int kTileBits = 13;
constexpr int kTileSpan = 1 << kTileBits;  // rows of a row block at most, columns of a chunk
constexpr int kTileThreads = 1024;
constexpr int kTileDirect = 2048;          // tiles with fewer entries gather from global memory
constexpr int kAdjGroupRows = 1 << 15;     // rows per adjoint workgroup at most (bounds the terms of one accumulator)
constexpr int kThreads = 256;

// One thread. Row blocks: consecutive rows, at most kTileSpan of them and (if more than one row) at most `budget`
// entries; groups of consecutive row blocks for the adjoint: at most kAdjGroupRows rows and `gbudget` entries (if
// more than one block). mail[0] = number of row blocks (-1: more than max_blocks), mail[1] = number of groups.
__global__ void tile_blocks_kernel(const int32_t* off, int64_t rows, int64_t budget, int64_t gbudget, int32_t max_blocks,
                                   int32_t* rb_start, int32_t* ga_start, int64_t* mail) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  int32_t nb = 0;
  int64_t s = 0;
  while (s < rows && nb < max_blocks) {
    int64_t hi = s + kTileSpan < rows ? s + kTileSpan : rows;
    if ((int64_t)off[hi] - off[s] > budget) {
      int64_t lo = s + 1, h2 = hi;  // largest end in [s+1, hi] within the budget (s+1 if none)
      while (lo < h2) {
        const int64_t mid = (lo + h2 + 1) / 2;
        if ((int64_t)off[mid] - off[s] <= budget) lo = mid;
        else h2 = mid - 1;
      }
      hi = lo;
    }
    rb_start[nb++] = (int32_t)s;
    s = hi;
  }
  rb_start[nb] = (int32_t)rows;
  if (s < rows) {
    mail[0] = -1;
    mail[1] = 0;
    return;
  }
  int32_t g = 0, b = 0;
  while (b < nb) {
    ga_start[g++] = b;
    int64_t r = 0, e = 0;
    do {
      r += rb_start[b + 1] - rb_start[b];
      e += (int64_t)off[rb_start[b + 1]] - off[rb_start[b]];
      ++b;
    } while (b < nb && r + (rb_start[b + 1] - rb_start[b]) <= kAdjGroupRows &&
             e + ((int64_t)off[rb_start[b + 1]] - off[rb_start[b]]) <= gbudget);
  }
  ga_start[g] = nb;
  mail[0] = nb;
  mail[1] = g;
}

__device__ __forceinline__ int block_of_row(const int32_t* rb_start, int nrb, int64_t r) {
  int lo = 0, hi = nrb - 1;  // last block whose first row is <= r
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (rb_start[mid] <= r) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}

// One wave per row; the columns of a row ascend, so the lanes of a 64-entry step that fall into one chunk are a run:
// the first lane of each run adds the run's length to its tile's counter (FILL: takes that many slots from the tile's
// cursor and the lanes of the run write their entries there).
template <bool FILL>
__global__ __launch_bounds__(kThreads) void tile_scatter_kernel(const int32_t* off, const int32_t* idx, int64_t rows, int32_t nrb,
                                                                int32_t ncb, const int32_t* rb_start, int32_t* counter,
                                                                const int32_t* tile_off, uint32_t* ent) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t r = wave; r < rows; r += nwaves) {
    const int rb = block_of_row(rb_start, nrb, r);
    const uint32_t rl = (uint32_t)(r - rb_start[rb]);
    const int32_t a = off[r], b = off[r + 1];
    for (int32_t e0 = a; e0 < b; e0 += 64) {
      const int32_t e = e0 + lane;
      const bool valid = e < b;
      const int32_t col = valid ? idx[e] : -1;
      const int32_t ch = valid ? (col >> kTileBits) : -1;
      const int32_t prev = __shfl_up(ch, 1, 64);
      const bool head = valid && (lane == 0 || ch != prev);
      const uint64_t heads = __ballot(head);
      const int nvalid = __popcll(__ballot(valid));
      int32_t base = 0;
      if (head) {
        const uint64_t above = lane == 63 ? 0ull : heads >> (lane + 1);
        const int len = above ? (__ffsll((long long)above)) : (nvalid - lane);
        base = atomicAdd(&counter[(int64_t)rb * ncb + ch], len);
      }
      if (FILL) {
        const uint64_t upto = heads & (lane == 63 ? ~0ull : ((2ull << lane) - 1ull));   // heads at or below this lane
        const int headlane = valid ? 63 - __clzll((long long)upto) : 0;
        const int32_t hb = __shfl(base, headlane, 64);
        if (valid) ent[(int64_t)tile_off[(int64_t)rb * ncb + ch] + hb + (lane - headlane)] = (rl << kTileBits) | (uint32_t)(col & (kTileSpan - 1));
      }
    }
  }
}

// The fill leaves the entries of a tile row by row: 64 consecutive entries would share a row, and the forward
// product's 64 lanes one accumulator. Position p of the tile takes the entry at (p * step) mod m instead, step about
// m/61 and coprime to m: neighbouring lanes then hold entries of different rows and columns in both products.
__global__ __launch_bounds__(kThreads) void tile_shuffle_kernel(const int32_t* tile_off, int64_t tiles, const uint32_t* in, uint32_t* out) {
  for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
    const int32_t e0 = tile_off[t];
    const uint32_t m = (uint32_t)(tile_off[t + 1] - e0);
    if (m == 0) continue;
    uint32_t step = m / 61 + 1;
    for (;; ++step) {  // the next value coprime to m (m + 1 at the latest)
      uint32_t x = step, y = m;
      while (y) {
        const uint32_t r = x % y;
        x = y;
        y = r;
      }
      if (x == 1) break;
    }
    for (uint32_t p = threadIdx.x; p < m; p += blockDim.x) out[e0 + p] = in[e0 + (uint32_t)(((uint64_t)p * step) % m)];
  }
}

struct TileArgs {
  int64_t rows, cols;
  int32_t nrb, ncb, cpg;
  const int32_t *rb_start, *ga_start, *tile_off;
  const uint32_t* ent;
  const long long* q;  // the source vector as integers (forward: cols entries, adjoint: rows entries)
  int sh;              // low bits dropped from them (rounded)
  long long* partial;  // forward: [chunk groups][rows]; adjoint: [row-block groups][cols]
};

__device__ __forceinline__ long long drop_bits(long long q, int sh) { return sh ? (q + (1ll << (sh - 1))) >> sh : q; }

template <bool ADJ>
__global__ __launch_bounds__(kTileThreads) void tile_spmv_kernel(TileArgs a) {
  extern __shared__ long long tile_smem[];
  long long* acc = tile_smem;            // [kTileSpan] target piece
  long long* src = tile_smem + kTileSpan;  // [kTileSpan] source piece
  const int tid = threadIdx.x;
  for (int i = tid; i < kTileSpan; i += kTileThreads) acc[i] = 0;
  __syncthreads();
  // forward: x = row block, y = chunk group, walks chunks; adjoint: x = chunk, y = row-block group, walks row blocks
  const int fixed = blockIdx.x;
  const int w_begin = ADJ ? a.ga_start[blockIdx.y] : (int)blockIdx.y * a.cpg;
  int w_end = ADJ ? a.ga_start[blockIdx.y + 1] : w_begin + a.cpg;
  if (!ADJ && w_end > a.ncb) w_end = a.ncb;
  bool staged = false;
  for (int w = w_begin; w < w_end; ++w) {
    const int rb = ADJ ? w : fixed, cb = ADJ ? fixed : w;
    const int64_t t = (int64_t)rb * a.ncb + cb;
    const int32_t e0 = a.tile_off[t], e1 = a.tile_off[t + 1];
    if (e0 == e1) continue;
    // source piece: forward = columns of the chunk, adjoint = rows of the block
    const int64_t s0 = ADJ ? (int64_t)a.rb_start[rb] : (int64_t)cb * kTileSpan;
    const int64_t s_end = ADJ ? (int64_t)a.rb_start[rb + 1] : (s0 + kTileSpan < a.cols ? s0 + kTileSpan : a.cols);
    const long long* qs = a.q + s0;
    const bool direct = e1 - e0 < kTileDirect;
    if (!direct) {
      if (staged) __syncthreads();  // the piece staged before is no longer read
      const int len = (int)(s_end - s0);
      for (int i = tid; i < len; i += kTileThreads) src[i] = drop_bits(qs[i], a.sh);
      __syncthreads();
      staged = true;
    }
    int32_t e = e0 + tid;
    for (; e + 3 * kTileThreads < e1; e += 4 * kTileThreads) {  // four entries in flight
      uint32_t v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = a.ent[e + u * kTileThreads];
      long long val[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t si = ADJ ? (v[u] >> kTileBits) : (v[u] & (kTileSpan - 1));
        val[u] = direct ? drop_bits(qs[si], a.sh) : src[si];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t ti = ADJ ? (v[u] & (kTileSpan - 1)) : (v[u] >> kTileBits);
        atomicAdd((unsigned long long*)&acc[ti], (unsigned long long)val[u]);
      }
    }
    for (; e < e1; e += kTileThreads) {
      const uint32_t v = a.ent[e];
      const uint32_t si = ADJ ? (v >> kTileBits) : (v & (kTileSpan - 1));
      const uint32_t ti = ADJ ? (v & (kTileSpan - 1)) : (v >> kTileBits);
      const long long val = direct ? drop_bits(qs[si], a.sh) : src[si];
      atomicAdd((unsigned long long*)&acc[ti], (unsigned long long)val);
    }
  }
  __syncthreads();
  const int64_t t0 = ADJ ? (int64_t)fixed * kTileSpan : (int64_t)a.rb_start[fixed];
  const int64_t t_end = ADJ ? (t0 + kTileSpan < a.cols ? t0 + kTileSpan : a.cols) : (int64_t)a.rb_start[fixed + 1];
  const int64_t span = ADJ ? a.cols : a.rows;
  long long* out = a.partial + (int64_t)blockIdx.y * span + t0;
  for (int i = tid; i < (int)(t_end - t0); i += kTileThreads) out[i] = acc[i];
}

// out[i] = scal[0] * 2^sh * sum over the groups of partial[g][i]; the groups are added as two 32-bit halves so that
// the total may exceed 63 bits
__global__ __launch_bounds__(256) void tile_reduce_kernel(const long long* partial, int64_t len, int groups, const double* scal, int sh,
                                                          double* out, unsigned long long* slot) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0 && slot) *slot = 0ull;
  if (i >= len) return;
  out[i] = ds_tile_sum(partial, len, groups, sh, i) * scal[0];
}

int ceil_log2(int64_t v) {
  int b = 0;
  while (((int64_t)1 << b) < v) ++b;
  return b;
}
}  // namespace

static void tile_shape(const ds_ctx* ctx, int64_t rows, int64_t cols, int64_t nnz, int64_t* budget, int64_t* gbudget,
                       int32_t* max_blocks, int32_t* ncb) {
  *ncb = (int32_t)((cols + kTileSpan - 1) / kTileSpan);
  // entry-heavy row blocks: 16, or more where the matrix has few column chunks (the adjoint product runs one
  // workgroup per chunk and group of row blocks, and wants two per compute unit)
  int64_t parts = (2 * (int64_t)ctx->num_cus + *ncb - 1) / *ncb;
  if (parts < 16) parts = 16;
  if (parts > 64) parts = 64;
  *budget = nnz / parts > 65536 ? nnz / parts : 65536;
  *gbudget = parts > 16 ? *budget : (nnz / 6 > 4 * *budget ? nnz / 6 : 4 * *budget);
  *max_blocks = (int32_t)(rows / kTileSpan + 2 * (nnz / *budget) + 8);
}

size_t ds_tile_ws_bytes(const ds_ctx* ctx, int64_t rows, int64_t cols, int64_t nnz) {
  int64_t budget, gbudget;
  int32_t max_blocks, ncb;
  tile_shape(ctx, rows, cols, nnz, &budget, &gbudget, &max_blocks, &ncb);
  const size_t tiles = (size_t)max_blocks * ncb + 2;
  // forward partials: at most 32 chunk groups of `rows`; adjoint: at most max_blocks groups, in practice
  // a few more than rows / 32768, of `cols`
  return 2 * ds_align((max_blocks + 2) * 4) + 2 * ds_align(tiles * 4) + ds_align((size_t)(nnz + 1) * 4) +
         ds_align((size_t)32 * rows * 8) + ds_align((size_t)(2 * (rows / kAdjGroupRows) + 2 * 64 + 24) * cols * 8) + ds_scan_arena_bytes((int64_t)tiles) +
         4096;
}

int ds_tile_build(ds_ctx* ctx, int64_t rows, int64_t cols, int64_t nnz, int64_t max_row_size, const int32_t* off,
                  int32_t* idx, void* ws, ds_tile_plan* plan) {
  hipStream_t st = ctx->stream;
  memset(plan, 0, sizeof(*plan));
  plan->rows = rows;
  plan->cols = cols;
  plan->nnz = nnz;
  if (rows <= 0 || nnz <= 0) return DS_OK;
  int64_t budget, gbudget;
  int32_t max_blocks, ncb;
  tile_shape(ctx, rows, cols, nnz, &budget, &gbudget, &max_blocks, &ncb);
  plan->ncb = ncb;
  char* p = (char*)ws;
  auto take = [&](size_t bytes) {
    char* q = p;
    p += ds_align(bytes);
    return q;
  };
  plan->rb_start = (int32_t*)take((max_blocks + 2) * 4);
  plan->ga_start = (int32_t*)take((max_blocks + 2) * 4);
  const size_t tiles_max = (size_t)max_blocks * ncb + 2;
  int32_t* counter = (int32_t*)take(tiles_max * 4);
  plan->tile_off = (int32_t*)take(tiles_max * 4);
  plan->ent = (uint32_t*)take((size_t)(nnz + 1) * 4);
  hipLaunchKernelGGL(tile_blocks_kernel, dim3(1), dim3(64), 0, st, off, rows, budget, gbudget, max_blocks, plan->rb_start,
                     plan->ga_start, ctx->d_mail + 4);
  DS_HIP(ctx, hipGetLastError());
  DS_TRY(ds_mail_fetch(ctx, 8));
  if (ctx->h_mail[4] <= 0) return ds_fail(ctx, DS_EINTERNAL, "index tiles: more row blocks than planned (%d)", max_blocks);
  plan->nrb = (int32_t)ctx->h_mail[4];
  plan->nga = (int32_t)ctx->h_mail[5];
  if (plan->nga > 2 * (rows / kAdjGroupRows) + 2 * 64 + 24)
    return ds_fail(ctx, DS_EINTERNAL, "index tiles: %d adjoint groups, %lld planned", plan->nga, (long long)(2 * (rows / kAdjGroupRows) + 152));
  const int64_t tiles = (int64_t)plan->nrb * ncb;
  // forward: (row block, chunk group) workgroups, about three per compute unit
  int32_t gf = (int32_t)((3 * (int64_t)ctx->num_cus + plan->nrb - 1) / plan->nrb);
  if (gf > 32) gf = 32;
  if (gf > ncb) gf = ncb;
  if (gf < 1) gf = 1;
  plan->cpg = (ncb + gf - 1) / gf;
  plan->gf = (ncb + plan->cpg - 1) / plan->cpg;
  const size_t pf = (size_t)plan->gf * rows * 8, pa = (size_t)plan->nga * cols * 8;
  plan->partial = (long long*)take(pf > pa ? pf : pa);
  // terms of one accumulator: forward at most max_row_size, adjoint at most the rows of a group; the integers are
  // below 2^54 in magnitude
  const int64_t rows_per_group = kAdjGroupRows > kTileSpan ? kAdjGroupRows : kTileSpan;
  plan->sh_f = ceil_log2(max_row_size > 1 ? max_row_size : 1) - 8;
  plan->sh_a = ceil_log2(rows_per_group < rows ? rows_per_group : rows) - 8;
  if (plan->sh_f < 0) plan->sh_f = 0;
  if (plan->sh_a < 0) plan->sh_a = 0;
  int64_t blocks = (rows * 64 + kThreads - 1) / kThreads;
  if (blocks > (int64_t)ctx->num_cus * 16) blocks = (int64_t)ctx->num_cus * 16;
  DS_HIP(ctx, hipMemsetAsync(counter, 0, (tiles + 1) * 4, st));
  hipLaunchKernelGGL(tile_scatter_kernel<false>, dim3((unsigned)blocks), dim3(kThreads), 0, st, off, idx, rows, plan->nrb, ncb,
                     plan->rb_start, counter, (const int32_t*)nullptr, (uint32_t*)nullptr);
  DS_HIP(ctx, hipGetLastError());
  // the scan's scratch comes from the context's arena, after everything the caller holds
  DS_TRY(ds_scan_exclusive_i32(ctx, counter, plan->tile_off, tiles + 1, nullptr));
  DS_HIP(ctx, hipMemsetAsync(counter, 0, (tiles + 1) * 4, st));
  hipLaunchKernelGGL(tile_scatter_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, st, off, idx, rows, plan->nrb, ncb,
                     plan->rb_start, counter, plan->tile_off, plan->ent);
  DS_HIP(ctx, hipGetLastError());
  // the index lists are not needed any more: their memory takes the entries in their final order
  hipLaunchKernelGGL(tile_shuffle_kernel, dim3((unsigned)(tiles < 65536 ? tiles : 65536)), dim3(kThreads), 0, st, plan->tile_off, tiles,
                     plan->ent, (uint32_t*)idx);
  DS_HIP(ctx, hipGetLastError());
  plan->ent = (uint32_t*)idx;
  const int lds = 2 * kTileSpan * 8;
  DS_HIP(ctx, hipFuncSetAttribute((const void*)tile_spmv_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  DS_HIP(ctx, hipFuncSetAttribute((const void*)tile_spmv_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
  return DS_OK;
}

int ds_tile_spmv(ds_ctx* ctx, const ds_tile_plan* p, int adjoint, const long long* q64, const double* scal, double* out,
                 int clear_slot) {
  if (p->rows <= 0) return DS_OK;
  if (p->nnz <= 0) {  // rows without a single entry (the empty coalition of pair 0): a zero result
    if (out) DS_HIP(ctx, hipMemsetAsync(out, 0, (size_t)(adjoint ? p->cols : p->rows) * 8, ctx->stream));
    if (clear_slot) DS_HIP(ctx, hipMemsetAsync((void*)(scal + 1), 0, 8, ctx->stream));
    return DS_OK;
  }
  TileArgs a;
  a.rows = p->rows;
  a.cols = p->cols;
  a.nrb = p->nrb;
  a.ncb = p->ncb;
  a.cpg = p->cpg;
  a.rb_start = p->rb_start;
  a.ga_start = p->ga_start;
  a.tile_off = p->tile_off;
  a.ent = p->ent;
  a.q = q64;
  a.partial = p->partial;
  const int lds = 2 * kTileSpan * 8;
  unsigned long long* slot = clear_slot ? (unsigned long long*)(scal + 1) : (unsigned long long*)nullptr;
  if (!adjoint) {
    a.sh = p->sh_f;
    hipLaunchKernelGGL(tile_spmv_kernel<false>, dim3((unsigned)p->nrb, (unsigned)p->gf), dim3(kTileThreads), lds, ctx->stream, a);
    if (out)
      hipLaunchKernelGGL(tile_reduce_kernel, dim3((unsigned)((p->rows + 255) / 256)), dim3(256), 0, ctx->stream, p->partial,
                         p->rows, (int)p->gf, scal, p->sh_f, out, slot);
  } else {
    a.sh = p->sh_a;
    hipLaunchKernelGGL(tile_spmv_kernel<true>, dim3((unsigned)p->ncb, (unsigned)p->nga), dim3(kTileThreads), lds, ctx->stream, a);
    if (out)
      hipLaunchKernelGGL(tile_reduce_kernel, dim3((unsigned)((p->cols + 255) / 256)), dim3(256), 0, ctx->stream, p->partial,
                         p->cols, (int)p->nga, scal, p->sh_a, out, slot);
  }
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}
