// k-hop computational-graph extraction on the device.
//
// Paper, "Computational graph": an L-layer GNN's prediction for v depends only on
// v's 1..L-hop neighbours and the edges among them; that induced sub-graph G_c(v)
// is what the explanation works on, and its edges are the players. The steps here:
// level-synchronous BFS along CSR rows (in-neighbours), local ids in ascending
// (hop, global id) order by prefix sums, induced sub-CSR by ordered wave
// compaction, player ids in ascending global (a, b) order, and a gather of the
// feature rows.
#include "internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kScanItems = 8;                       // per thread
constexpr int kScanTile = kThreads * kScanItems;    // per block

// ---------------- exclusive prefix sum (int32), three phases ----------------

__device__ __forceinline__ int block_reduce_sum(int v, int* sh) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  int total = 0;
  for (int i = 0; i < kThreads / 64; ++i) total += sh[i];
  __syncthreads();
  return total;
}

__global__ __launch_bounds__(kThreads) void scan_tile_sums(const int32_t* in, int64_t count, int32_t* tile_sums) {
  __shared__ int sh[kThreads / 64];
  const int64_t base = (int64_t)blockIdx.x * kScanTile;
  int s = 0;
  for (int i = 0; i < kScanItems; ++i) {
    const int64_t idx = base + (int64_t)i * kThreads + threadIdx.x;
    if (idx < count) s += in[idx];
  }
  const int total = block_reduce_sum(s, sh);
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

// single block: exclusive scan of the tile sums in place; total -> mail slot
__global__ __launch_bounds__(kThreads) void scan_tile_offsets(int32_t* tile_sums, int64_t tiles, int64_t* total_out) {
  __shared__ int sh[kThreads];
  __shared__ long long carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int64_t base = 0; base < tiles; base += kThreads) {
    const int64_t idx = base + threadIdx.x;
    const int v = idx < tiles ? tile_sums[idx] : 0;
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int o = 1; o < kThreads; o <<= 1) {  // Hillis-Steele inclusive scan
      int add = threadIdx.x >= o ? sh[threadIdx.x - o] : 0;
      __syncthreads();
      sh[threadIdx.x] += add;
      __syncthreads();
    }
    const long long c = carry;
    if (idx < tiles) tile_sums[idx] = (int32_t)(c + sh[threadIdx.x] - v);
    __syncthreads();
    if (threadIdx.x == kThreads - 1) carry = c + sh[kThreads - 1];
    __syncthreads();
  }
  if (threadIdx.x == 0 && total_out) *total_out = carry;
}

__global__ __launch_bounds__(kThreads) void scan_apply(const int32_t* in, int32_t* out, int64_t count,
                                                       const int32_t* tile_offsets) {
  __shared__ int sh[kThreads];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int v[kScanItems];
  int s = 0;
  for (int i = 0; i < kScanItems; ++i) {
    v[i] = (base + i < count) ? in[base + i] : 0;
    s += v[i];
  }
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int o = 1; o < kThreads; o <<= 1) {
    int add = threadIdx.x >= o ? sh[threadIdx.x - o] : 0;
    __syncthreads();
    sh[threadIdx.x] += add;
    __syncthreads();
  }
  int run = tile_offsets[blockIdx.x] + sh[threadIdx.x] - s;
  for (int i = 0; i < kScanItems; ++i) {
    if (base + i < count) out[base + i] = run;
    run += v[i];
  }
}

// short inputs: the whole exclusive scan in one launch. Every thread owns a contiguous run of items: it sums
// them, the 1024 run sums are scanned in LDS, and the thread then walks its run again (out may alias in: a
// run is read and written by its owner only, after every first pass is over).
constexpr int kSmallScanThreads = 1024;
constexpr int64_t kSmallScanMax = 4096;  // beyond a few items per thread the strided runs cost more than two extra launches
__global__ __launch_bounds__(kSmallScanThreads) void scan_small_kernel(const int32_t* in, int32_t* out, int64_t count,
                                                                       int64_t* total_out) {
  __shared__ int sh[kSmallScanThreads];
  const int tid = threadIdx.x;
  const int64_t per = (count + kSmallScanThreads - 1) / kSmallScanThreads;
  const int64_t b = (int64_t)tid * per, e = b + per < count ? b + per : count;
  int s = 0;
  for (int64_t i = b; i < e; ++i) s += in[i];
  sh[tid] = s;
  __syncthreads();
  for (int o = 1; o < kSmallScanThreads; o <<= 1) {  // Hillis-Steele inclusive scan of the run sums
    const int add = tid >= o ? sh[tid - o] : 0;
    __syncthreads();
    sh[tid] += add;
    __syncthreads();
  }
  int run = sh[tid] - s;
  for (int64_t i = b; i < e; ++i) {
    const int v = in[i];
    out[i] = run;
    run += v;
  }
  if (tid == kSmallScanThreads - 1 && total_out) *total_out = sh[tid];
}

}  // namespace

size_t ds_scan_arena_bytes(int64_t count) {
  const int64_t tiles = (count + kScanTile - 1) / kScanTile;
  return ds_align((tiles + 1) * sizeof(int32_t));
}

// out may alias in. The grand total goes to mail slot `total_mail_slot` (device side) if not null.
int ds_scan_exclusive_i32(ds_ctx* ctx, const int32_t* in, int32_t* out, int64_t count, int64_t* total_mail_slot) {
  if (count <= 0) {
    if (total_mail_slot) DS_HIP(ctx, hipMemsetAsync(total_mail_slot, 0, sizeof(int64_t), ctx->stream));
    return DS_OK;
  }
  if (count <= kSmallScanMax) {
    hipLaunchKernelGGL(scan_small_kernel, dim3(1), dim3(kSmallScanThreads), 0, ctx->stream, in, out, count, total_mail_slot);
    DS_HIP(ctx, hipGetLastError());
    return DS_OK;
  }
  const int64_t tiles = (count + kScanTile - 1) / kScanTile;
  int32_t* tile_sums = (int32_t*)ds_arena_alloc(ctx, (tiles + 1) * sizeof(int32_t));
  if (!tile_sums) return ds_fail(ctx, DS_EINTERNAL, "scan: arena exhausted");
  hipLaunchKernelGGL(scan_tile_sums, dim3((unsigned)tiles), dim3(kThreads), 0, ctx->stream, in, count, tile_sums);
  hipLaunchKernelGGL(scan_tile_offsets, dim3(1), dim3(kThreads), 0, ctx->stream, tile_sums, tiles, total_mail_slot);
  hipLaunchKernelGGL(scan_apply, dim3((unsigned)tiles), dim3(kThreads), 0, ctx->stream, in, out, count, tile_sums);
  DS_HIP(ctx, hipGetLastError());
  return DS_OK;
}

namespace {

// ---------------- CSR validation ----------------
__global__ void validate_csr_kernel(const int64_t* row_ptr, const int32_t* col, int64_t N, int64_t nnz, int* bad) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t i = wave; i < N; i += nwaves) {
    const int64_t a = row_ptr[i], b = row_ptr[i + 1];
    if (a > b || a < 0 || b > nnz) {
      if (lane == 0) atomicExch(bad, 1);
      continue;
    }
    for (int64_t e = a + lane; e < b; e += 64) {
      const int32_t c = col[e];
      if (c < 0 || c >= N || (e > a && col[e - 1] >= c)) atomicExch(bad, 2);
    }
  }
}

// ---------------- BFS ----------------
__global__ void fill_i32(int32_t* p, int64_t count, int32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) p[i] = v;
}

// mail layout (int64 slots): [0..7] level counts, [8] nnz_c, [9] players, [10] error, [11] members
__global__ void bfs_seed(int32_t* dist, int32_t* frontier, int64_t* mail, int64_t target) {
  dist[target] = 0;
  frontier[0] = (int32_t)target;
  for (int i = 0; i < 16; ++i) mail[i] = 0;
  mail[0] = 1;
}

__global__ __launch_bounds__(kThreads) void bfs_visit(const int64_t* row_ptr, const int32_t* col, int32_t* dist,
                                                      const int32_t* frontier, int32_t* next, int64_t* mail, int level) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const int64_t count = mail[level - 1];
  unsigned long long* next_count = (unsigned long long*)&mail[level];
  for (int64_t f = wave; f < count; f += nwaves) {
    const int64_t i = frontier[f];
    const int64_t a = row_ptr[i], b = row_ptr[i + 1];
    for (int64_t e = a + lane; e < b; e += 64) {
      const int32_t j = col[e];
      if (atomicCAS(&dist[j], -1, level) == -1) {
        const unsigned long long pos = atomicAdd(next_count, 1ull);
        next[pos] = j;
      }
    }
  }
}

// flags over the expanded index space h*N + g (local order = hop, then global id)
__global__ void member_flags(const int32_t* dist, int64_t N, int levels, int32_t* level_flag, int32_t* member_flag) {
  const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= N) return;
  const int d = dist[g];
  member_flag[g] = d >= 0 ? 1 : 0;
  for (int h = 0; h < levels; ++h) level_flag[(int64_t)h * N + g] = (d == h) ? 1 : 0;
}

struct GraphOut {
  int32_t* row_ptr;
  int32_t* col;
  int32_t* eid;
  int2* pl;
  int64_t* node_gid;
  int32_t* hop;
};

__global__ void assign_nodes(const int32_t* dist, const int32_t* lid_scan, const int32_t* rank_scan, int64_t N,
                             int64_t* node_gid, int32_t* hop, int32_t* lid_of_rank) {
  const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= N) return;
  const int d = dist[g];
  if (d < 0) return;
  const int32_t lid = lid_scan[(int64_t)d * N + g];
  node_gid[lid] = g;
  hop[lid] = d;
  lid_of_rank[rank_scan[g]] = lid;
}

// one wave per member (in global-id rank order): count induced entries and upper entries
__global__ __launch_bounds__(kThreads) void count_entries(const int64_t* row_ptr, const int32_t* col, const int32_t* dist,
                                                          const int64_t* node_gid, const int32_t* lid_of_rank, int64_t V,
                                                          int32_t* cnt_all_lid, int32_t* cnt_all_rank, int32_t* cnt_up_rank) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t rk = wave; rk < V; rk += nwaves) {
    const int32_t lid = lid_of_rank[rk];
    const int64_t g = node_gid[lid];
    const int64_t a = row_ptr[g], b = row_ptr[g + 1];
    int all = 0, up = 0;
    for (int64_t e = a + lane; e < b; e += 64) {
      const int32_t j = col[e];
      if (j != g && dist[j] >= 0) {
        ++all;
        if (j > g) ++up;
      }
    }
    for (int o = 32; o > 0; o >>= 1) {
      all += __shfl_down(all, o, 64);
      up += __shfl_down(up, o, 64);
    }
    if (lane == 0) {
      cnt_all_lid[lid] = all;
      cnt_all_rank[rk] = all;
      cnt_up_rank[rk] = up;
    }
  }
}

// one wave per member: ordered compaction of its row into the local CSR, player ids
// for the entries this row owns (undirected: neighbours with larger global id;
// directed: every entry).
__global__ __launch_bounds__(kThreads) void fill_entries(const int64_t* row_ptr, const int32_t* col, const int32_t* dist,
                                                         const int32_t* lid_scan, int64_t N, const int32_t* lid_of_rank,
                                                         const int32_t* player_start_rank, int64_t V, int directed,
                                                         GraphOut out) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int64_t rk = wave; rk < V; rk += nwaves) {
    const int32_t lid = lid_of_rank[rk];
    const int64_t g = out.node_gid[lid];
    const int64_t a = row_ptr[g], b = row_ptr[g + 1];
    int32_t pos = out.row_ptr[lid];
    int32_t ppos = player_start_rank[rk];
    for (int64_t e0 = a; e0 < b; e0 += 64) {
      const int64_t e = e0 + lane;
      int32_t j = -1, d = -1;
      if (e < b) {
        j = col[e];
        d = dist[j];
      }
      const bool in = (j >= 0) && (j != g) && (d >= 0);
      const bool own = in && (directed || j > g);
      const unsigned long long m_in = __ballot(in), m_own = __ballot(own);
      if (in) {
        const int32_t jl = lid_scan[(int64_t)d * N + j];
        const int32_t at = pos + __popcll(m_in & lt);
        out.col[at] = jl;
        int32_t p = -1;
        if (own) {
          p = ppos + __popcll(m_own & lt);
          out.pl[p] = directed ? make_int2(jl, lid) : make_int2(lid, jl);
        }
        out.eid[at] = p;
      }
      pos += __popcll(m_in);
      ppos += __popcll(m_own);
    }
  }
}

// undirected: entries (row b, neighbour a) with gid(a) < gid(b) look their player
// up in a's owned range (ascending in the global id of the far end).
__global__ void backfill_entries(GraphOut out, const int32_t* rank_scan, const int32_t* player_start_rank, int64_t V,
                                 int64_t* mail) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  for (int64_t t = wave; t < V; t += nwaves) {
    const int64_t g = out.node_gid[t];
    for (int32_t e = out.row_ptr[t] + lane; e < out.row_ptr[t + 1]; e += 64) {
      if (out.eid[e] >= 0) continue;
      const int32_t al = out.col[e];
      const int64_t ag = out.node_gid[al];
      const int32_t rk = rank_scan[ag];
      int32_t lo = player_start_rank[rk], hi = player_start_rank[rk + 1];
      int32_t found = -1;
      while (lo < hi) {
        const int32_t mid = (lo + hi) >> 1;
        const int64_t bg = out.node_gid[out.pl[mid].y];
        if (bg == g) {
          found = mid;
          break;
        }
        if (bg < g) lo = mid + 1; else hi = mid;
      }
      if (found < 0) atomicExch((unsigned long long*)&mail[10], 1ull);
      out.eid[e] = found < 0 ? 0 : found;
    }
  }
}

__global__ void gather_rows(const float* X, const int64_t* node_gid, int64_t V, int d0, float* Xc) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= V * d0) return;
  const int64_t t = idx / d0;
  const int f = (int)(idx - t * d0);
  Xc[idx] = X[node_gid[t] * d0 + f];
}

inline unsigned blocks_for(int64_t n, int per = kThreads) { return (unsigned)((n + per - 1) / per); }

}  // namespace

int ds_validate_csr(ds_ctx* ctx) {
  ds_arena_reset(ctx);
  DS_TRY(ds_arena_reserve(ctx, 4096));
  int* bad = (int*)ds_arena_alloc(ctx, 256);
  DS_HIP(ctx, hipMemsetAsync(bad, 0, sizeof(int), ctx->stream));
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail, ctx->row_ptr, sizeof(int64_t), hipMemcpyDeviceToHost, ctx->stream));
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail + 1, ctx->row_ptr + ctx->N, sizeof(int64_t), hipMemcpyDeviceToHost, ctx->stream));
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  if (ctx->h_mail[0] != 0 || ctx->h_mail[1] < 0)
    return ds_fail(ctx, DS_EINVAL, "row_ptr[0] must be 0 and row_ptr[N] >= 0");
  ctx->nnz = ctx->h_mail[1];
  if (ctx->N > 0) {
    hipLaunchKernelGGL(validate_csr_kernel, dim3(ctx->num_cus * 8), dim3(kThreads), 0, ctx->stream, ctx->row_ptr,
                       ctx->col, ctx->N, ctx->nnz, bad);
    DS_HIP(ctx, hipGetLastError());
  }
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail, bad, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  const int code = *(int*)ctx->h_mail;
  ds_arena_reset(ctx);
  if (code == 1) return ds_fail(ctx, DS_EINVAL, "row_ptr is not monotone within [0, nnz]");
  if (code == 2) return ds_fail(ctx, DS_EINVAL, "col has an id outside [0, N) or a row that is not strictly ascending");
  return DS_OK;
}

namespace {
__global__ void zero_three_kernel(int32_t* a, int32_t* b, int32_t* c) {
  if (threadIdx.x == 0) {
    *a = 0;
    *b = 0;
    *c = 0;
  }
}
// the three per-node arrays of the computational graph in one launch (row_ptr has V + 1 entries)
__global__ void copy_node_arrays_kernel(const int32_t* rp, const int64_t* gid, const int32_t* hop, int64_t V, int32_t* rp_out,
                                        int64_t* gid_out, int32_t* hop_out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i <= V) rp_out[i] = rp[i];
  if (i < V) {
    gid_out[i] = gid[i];
    hop_out[i] = hop[i];
  }
}
struct BallSizes { int32_t v[8]; };
// out[h] = row_ptr[ball[h]]: the CSR entries of the rows within h hops
__global__ void ball_entries_kernel(const int32_t* row_ptr, BallSizes b, int64_t* out) {
  if (threadIdx.x < 8) out[threadIdx.x] = row_ptr[b.v[threadIdx.x]];
}
}  // namespace

int ds_extract_impl(ds_ctx* ctx, int64_t target, int hops, int directed, ds_cgraph** out_cg) {
  if (!ctx->row_ptr) return ds_fail(ctx, DS_EINVAL, "ds_set_graph has not been called");
  if (!ctx->X) return ds_fail(ctx, DS_EINVAL, "ds_set_features has not been called");
  if (target < 0 || target >= ctx->N) return ds_fail(ctx, DS_EINVAL, "target %lld outside [0, %lld)", (long long)target, (long long)ctx->N);
  if (hops < 1 || hops > DS_MAX_HOPS) return ds_fail(ctx, DS_EINVAL, "hops must be in [1, %d]", DS_MAX_HOPS);
  const int64_t N = ctx->N;
  const int levels = hops + 1;
  hipStream_t st = ctx->stream;

  // phase 1 temporaries, all O(N)
  ds_arena_reset(ctx);
  size_t need = ds_align((N + 1) * 4) * 16 + ds_align((size_t)levels * N * 4) +
                ds_scan_arena_bytes((int64_t)levels * N) + 4 * ds_scan_arena_bytes(N + 1) + 65536;
  DS_TRY(ds_arena_reserve(ctx, need));
  int32_t* dist = (int32_t*)ds_arena_alloc(ctx, N * 4);
  int32_t* fr_a = (int32_t*)ds_arena_alloc(ctx, N * 4);
  int32_t* fr_b = (int32_t*)ds_arena_alloc(ctx, N * 4);
  int32_t* rank_scan = (int32_t*)ds_arena_alloc(ctx, N * 4);
  int32_t* lid_scan = (int32_t*)ds_arena_alloc(ctx, (size_t)levels * N * 4);
  if (!dist || !fr_a || !fr_b || !rank_scan || !lid_scan) return ds_fail(ctx, DS_EINTERNAL, "extract: arena exhausted");
  int64_t* mail = ctx->d_mail;

  hipLaunchKernelGGL(fill_i32, dim3(blocks_for(N)), dim3(kThreads), 0, st, dist, N, -1);
  hipLaunchKernelGGL(bfs_seed, dim3(1), dim3(1), 0, st, dist, fr_a, mail, target);
  int32_t *cur = fr_a, *nxt = fr_b;
  for (int h = 1; h <= hops; ++h) {
    hipLaunchKernelGGL(bfs_visit, dim3(ctx->num_cus * 4), dim3(kThreads), 0, st, ctx->row_ptr, ctx->col, dist, cur, nxt, mail, h);
    int32_t* t = cur; cur = nxt; nxt = t;
  }
  hipLaunchKernelGGL(member_flags, dim3(blocks_for(N)), dim3(kThreads), 0, st, dist, N, levels, lid_scan, rank_scan);
  DS_HIP(ctx, hipGetLastError());
  DS_TRY(ds_scan_exclusive_i32(ctx, lid_scan, lid_scan, (int64_t)levels * N, nullptr));
  DS_TRY(ds_scan_exclusive_i32(ctx, rank_scan, rank_scan, N, mail + 11));
  DS_TRY(ds_mail_fetch(ctx, 16));
  int64_t V = ctx->h_mail[11];
  int64_t ball[8] = {0};
  {
    int64_t acc = 0;
    for (int h = 0; h <= hops; ++h) {
      acc += ctx->h_mail[h];
      ball[h] = acc;
    }
    if (acc != V) return ds_fail(ctx, DS_EINTERNAL, "extract: level counts (%lld) disagree with member count (%lld)", (long long)acc, (long long)V);
  }
  if (V > 0x7ffffff0LL) return ds_fail(ctx, DS_EINVAL, "computational graph too large");

  // phase 2 temporaries, O(V) (frontier buffers are free again and reused)
  int64_t* node_gid_tmp = (int64_t*)ds_arena_alloc(ctx, V * 8);
  int32_t* hop_tmp = (int32_t*)ds_arena_alloc(ctx, V * 4);
  int32_t* lid_of_rank = (int32_t*)ds_arena_alloc(ctx, V * 4);
  int32_t* rowptr_tmp = (int32_t*)ds_arena_alloc(ctx, (V + 1) * 4);
  int32_t* cnt_all_rank = (int32_t*)ds_arena_alloc(ctx, (V + 1) * 4);
  int32_t* cnt_up_rank = (int32_t*)ds_arena_alloc(ctx, (V + 1) * 4);
  if (!node_gid_tmp || !hop_tmp || !lid_of_rank || !rowptr_tmp || !cnt_all_rank || !cnt_up_rank) {
    // grow and redo would invalidate live buffers; the reserve above is sized by N >= V, so add headroom instead
    return ds_fail(ctx, DS_EINTERNAL, "extract: arena exhausted (phase 2)");
  }
  hipLaunchKernelGGL(assign_nodes, dim3(blocks_for(N)), dim3(kThreads), 0, st, dist, lid_scan, rank_scan, N, node_gid_tmp, hop_tmp, lid_of_rank);
  hipLaunchKernelGGL(zero_three_kernel, dim3(1), dim3(64), 0, st, rowptr_tmp + V, cnt_all_rank + V, cnt_up_rank + V);
  const unsigned wave_blocks = (unsigned)((V * 64 + kThreads - 1) / kThreads < (int64_t)ctx->num_cus * 8 ? (V * 64 + kThreads - 1) / kThreads : (int64_t)ctx->num_cus * 8);
  hipLaunchKernelGGL(count_entries, dim3(wave_blocks), dim3(kThreads), 0, st, ctx->row_ptr, ctx->col, dist, node_gid_tmp, lid_of_rank, V, rowptr_tmp, cnt_all_rank, cnt_up_rank);
  DS_HIP(ctx, hipGetLastError());
  DS_TRY(ds_scan_exclusive_i32(ctx, rowptr_tmp, rowptr_tmp, V + 1, mail + 8));
  int32_t* player_start = directed ? cnt_all_rank : cnt_up_rank;
  DS_TRY(ds_scan_exclusive_i32(ctx, player_start, player_start, V + 1, mail + 9));
  {  // number of CSR entries in the rows of every ball (rows are ordered by hop): mailbox slots 40..47
    BallSizes bs;
    for (int h = 0; h < 8; ++h) bs.v[h] = (int32_t)ball[h <= hops ? h : hops];
    hipLaunchKernelGGL(ball_entries_kernel, dim3(1), dim3(64), 0, st, rowptr_tmp, bs, mail + 40);
    DS_HIP(ctx, hipGetLastError());
    DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail + 40, mail + 40, 8 * sizeof(int64_t), hipMemcpyDeviceToHost, st));
  }
  DS_TRY(ds_mail_fetch(ctx, 16));
  const int64_t nnz_c = ctx->h_mail[8];
  const int64_t n = ctx->h_mail[9];
  if (nnz_c > 0x7ffffff0LL) return ds_fail(ctx, DS_EINVAL, "computational graph has too many entries");
  if (!directed && nnz_c != 2 * n)
    return ds_fail(ctx, DS_EINVAL, "CSR is not symmetric inside the computational graph (entries %lld, pairs %lld): undirected players need both directions", (long long)nnz_c, (long long)n);

  // the computational graph itself: one allocation
  ds_cgraph* cg = new ds_cgraph();
  memset(cg, 0, sizeof(*cg));
  cg->owner = ctx;
  const int d0 = ctx->d0, d1 = ds_first_width(ctx);
  const int att_heads = ctx->model_kind == DS_MODEL_GAT && ctx->L > 0 ? ctx->gat.heads[0] : 0;
  size_t off = 0;
  auto carve = [&](size_t bytes) { size_t o = off; off += ds_align(bytes); return o; };
  const size_t o_rp = carve((V + 1) * 4), o_col = carve(nnz_c * 4 + 4), o_eid = carve(nnz_c * 4 + 4);
  const size_t o_pl = carve(n * 8 + 8), o_gid = carve(V * 8), o_hop = carve(V * 4);
  const size_t o_x = carve((size_t)V * d0 * 4), o_p = carve((size_t)V * (d1 > 0 ? d1 : 1) * 4);
  const size_t o_pred = carve(256);
  const size_t o_att = carve((size_t)V * att_heads * 8 + 8);
  if (ctx->cg_spare && ctx->cg_spare_bytes >= off) {
    cg->block = ctx->cg_spare;
    cg->block_bytes = ctx->cg_spare_bytes;
    ctx->cg_spare = nullptr;
    ctx->cg_spare_bytes = 0;
  } else {
    cg->block_bytes = off;
    if (hipMalloc(&cg->block, off) != hipSuccess) {
      (void)hipGetLastError();
      delete cg;
      return ds_fail(ctx, DS_ENOMEM, "extract: cannot allocate %zu bytes for the computational graph", off);
    }
  }
  char* base = (char*)cg->block;
  cg->row_ptr = (int32_t*)(base + o_rp);
  cg->col = (int32_t*)(base + o_col);
  cg->eid = (int32_t*)(base + o_eid);
  cg->pl = (int2*)(base + o_pl);
  cg->node_gid = (int64_t*)(base + o_gid);
  cg->hop = (int32_t*)(base + o_hop);
  cg->Xc = (float*)(base + o_x);
  cg->P = (float*)(base + o_p);
  cg->d_pred = (int32_t*)(base + o_pred);
  cg->att = (float*)(base + o_att);
  cg->pred_class = -1;
  cg->d0 = d0;
  cg->d1 = d1;
  cg->att_heads = att_heads;
  for (int h = 0; h < 8; ++h) cg->ball_entries[h] = ctx->h_mail[40 + h];
  cg->info.num_players = n;
  cg->info.num_nodes = V;
  cg->info.num_entries = nnz_c;
  cg->info.target = target;
  cg->info.hops = hops;
  cg->info.directed = directed;
  for (int h = 0; h < 8; ++h) cg->info.ball[h] = h <= hops ? ball[h] : ball[hops];
  ctx->graphs.push_back(cg);
  *out_cg = cg;

  hipLaunchKernelGGL(copy_node_arrays_kernel, dim3((unsigned)((V + 1 + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                     rowptr_tmp, node_gid_tmp, hop_tmp, V, cg->row_ptr, cg->node_gid, cg->hop);
  GraphOut go{cg->row_ptr, cg->col, cg->eid, cg->pl, cg->node_gid, cg->hop};
  hipLaunchKernelGGL(fill_entries, dim3(wave_blocks), dim3(kThreads), 0, st, ctx->row_ptr, ctx->col, dist, lid_scan, N, lid_of_rank, player_start, V, directed, go);
  if (!directed && nnz_c > 0)
    hipLaunchKernelGGL(backfill_entries, dim3(wave_blocks), dim3(kThreads), 0, st, go, rank_scan, player_start, V, mail);
  if (V * d0 > 0)
    hipLaunchKernelGGL(gather_rows, dim3(blocks_for(V * d0)), dim3(kThreads), 0, st, ctx->X, cg->node_gid, V, d0, cg->Xc);
  DS_HIP(ctx, hipGetLastError());
  DS_TRY(ds_mail_fetch(ctx, 16));
  ds_arena_reset(ctx);
  if (ctx->h_mail[10] != 0) {
    ds_cgraph_free(ctx, cg);
    *out_cg = nullptr;
    return ds_fail(ctx, DS_EINVAL, "CSR is not symmetric inside the computational graph: an entry has no reverse entry");
  }
  return DS_OK;
}
