// Top-k edge selection and the fidelity scores of an explanation.
//
// Paper, overview step 5 (rank the edges by Shapley value, keep the top k as the explanation
// sub-graph G_s) and the evaluation-metric section:
//   Fidelity+ = | f(G_c) - f(G_c \ G_s) |,   Fidelity- = | f(G_c) - f(G_s) |.
// Ranking is by descending phi, ties to the lower player index: player j gets the 64-bit key
// (order-preserving image of phi_j) << 32 | ~j, the k-th largest key is found by an 8-pass radix
// select (one workgroup per k), and the two mask rows (G_s and its complement) are emitted with
// wave ballots. The masked inference kernel then evaluates them like any other coalition.
#include "internal.h"

namespace {
constexpr int kSelThreads = 1024;

__device__ __forceinline__ uint64_t rank_key(float v, int64_t j) {
  uint32_t u = __float_as_uint(v + 0.0f);  // -0 ranks as +0
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger float -> larger unsigned
  return ((uint64_t)u << 32) | (uint32_t)(~(uint32_t)j);
}

// thr[t] = k-th largest key (0 -> every player selected; all-ones with flag none -> nobody)
__global__ __launch_bounds__(kSelThreads) void topk_threshold_kernel(const float* phi, int64_t n, const int64_t* ks,
                                                                     uint64_t* thr, int32_t* none) {
  __shared__ unsigned int hist[256];
  __shared__ uint64_t prefix_s;
  __shared__ int64_t want_s;
  const int t = blockIdx.x;
  int64_t k = ks[t];
  if (k <= 0) {
    if (threadIdx.x == 0) { thr[t] = ~0ull; none[t] = 1; }
    return;
  }
  if (k >= n) {
    if (threadIdx.x == 0) { thr[t] = 0ull; none[t] = 0; }
    return;
  }
  if (threadIdx.x == 0) { prefix_s = 0; want_s = k; }
  __syncthreads();
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
    for (int i = threadIdx.x; i < 256; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    const uint64_t prefix = prefix_s;
    const uint64_t himask = pass == 0 ? 0ull : (~0ull << (shift + 8));
    for (int64_t j = threadIdx.x; j < n; j += kSelThreads) {
      const uint64_t key = rank_key(phi[j], j);
      if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 0xFF], 1u);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int64_t want = want_s;
      int b = 255;
      while (b > 0 && (int64_t)hist[b] < want) { want -= hist[b]; --b; }
      prefix_s = prefix | ((uint64_t)b << shift);
      want_s = want;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) { thr[t] = prefix_s; none[t] = 0; }
}

// rows 2t (G_s) and 2t+1 (complement) of Z[2T x W]
__global__ void topk_masks_kernel(const float* phi, int64_t n, const uint64_t* thr, const int32_t* none, int T, uint64_t* Z) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const int64_t W = (n + 63) / 64;
  const uint64_t tail = (n & 63) ? ((1ull << (n & 63)) - 1ull) : ~0ull;
  for (int64_t item = wave; item < (int64_t)T * W; item += nwaves) {
    const int t = (int)(item / W);
    const int64_t wd = item - (int64_t)t * W;
    const int64_t j = wd * 64 + lane;
    const bool in = j < n && !none[t] && rank_key(phi[j], j) >= thr[t];
    const uint64_t word = __ballot(in);
    if (lane == 0) {
      Z[(2 * (int64_t)t) * W + wd] = word;
      Z[(2 * (int64_t)t + 1) * W + wd] = ~word & (wd == W - 1 ? tail : ~0ull);
    }
  }
}
}  // namespace

extern "C" int ds_fidelity(ds_ctx* ctx, const ds_cgraph* cg_in, const float* phi, const int64_t* topk, int32_t num_k,
                           int32_t score, float* fid_plus, float* fid_minus, uint64_t* masks_out) {
  if (!ctx || !cg_in) return DS_EINVAL;
  if (!phi || !topk || num_k < 1 || num_k > 4096 || !fid_plus || !fid_minus)
    return ds_fail(ctx, DS_EINVAL, "bad fidelity arguments");
  if (score != DS_SCORE_PROB && score != DS_SCORE_LOGIT) return ds_fail(ctx, DS_EINVAL, "unknown score %d", score);
  DS_HIP(ctx, hipSetDevice(ctx->device));
  ds_cgraph* cg = const_cast<ds_cgraph*>(cg_in);
  const int64_t n = cg->info.num_players, W = (n + 63) / 64;
  if (n < 1) return ds_fail(ctx, DS_EINVAL, "the computational graph has no players");
  const int64_t rows = 2 * (int64_t)num_k + 2;  // + the full and the empty coalition
  hipStream_t st = ctx->stream;
  ds_arena_reset(ctx);
  DS_TRY(ds_arena_reserve(ctx, ds_align(rows * W * 8) + ds_align(rows * 4) + 3 * ds_align(num_k * 8) +
                                   ds_eval_arena_bytes(ctx, cg, rows) + 4096));
  uint64_t* Z = (uint64_t*)ds_arena_alloc(ctx, rows * W * 8);
  float* y = (float*)ds_arena_alloc(ctx, rows * 4);
  int64_t* d_ks = (int64_t*)ds_arena_alloc(ctx, num_k * 8);
  uint64_t* d_thr = (uint64_t*)ds_arena_alloc(ctx, num_k * 8);
  int32_t* d_none = (int32_t*)ds_arena_alloc(ctx, num_k * 8);
  if (!Z || !y || !d_ks || !d_thr || !d_none) return ds_fail(ctx, DS_EINTERNAL, "fidelity: arena exhausted");
  DS_HIP(ctx, hipMemcpyAsync(d_ks, topk, num_k * 8, hipMemcpyHostToDevice, st));
  DS_HIP(ctx, hipStreamSynchronize(st));  // topk is pageable host memory owned by the caller
  hipLaunchKernelGGL(topk_threshold_kernel, dim3(num_k), dim3(kSelThreads), 0, st, phi, n, d_ks, d_thr, d_none);
  int64_t blocks = ((int64_t)num_k * W * 64 + 255) / 256;
  if (blocks > (int64_t)ctx->num_cus * 16) blocks = (int64_t)ctx->num_cus * 16;
  hipLaunchKernelGGL(topk_masks_kernel, dim3((unsigned)blocks), dim3(256), 0, st, phi, n, d_thr, d_none, num_k, Z);
  // last two rows: empty and full coalition (row 2T = empty, 2T+1 = full), same kernel with k = 0
  {
    int64_t* d_zero = d_ks;  // reuse after the threshold kernel has consumed it: stream-ordered
    DS_HIP(ctx, hipMemsetAsync(d_zero, 0, 8, st));
    hipLaunchKernelGGL(topk_threshold_kernel, dim3(1), dim3(kSelThreads), 0, st, phi, n, d_zero, d_thr, d_none);
    hipLaunchKernelGGL(topk_masks_kernel, dim3(16), dim3(256), 0, st, phi, n, d_thr, d_none, 1, Z + 2 * (int64_t)num_k * W);
  }
  DS_HIP(ctx, hipGetLastError());
  if (masks_out) DS_HIP(ctx, hipMemcpyAsync(masks_out, Z, 2 * (int64_t)num_k * W * 8, hipMemcpyDeviceToDevice, st));
  int rc = ds_eval_impl(ctx, cg, Z, rows, score, y, 0);
  if (rc != DS_OK) {
    ds_arena_reset(ctx);
    return rc;
  }
  std::vector<float> h(rows);
  DS_HIP(ctx, hipMemcpyAsync(h.data(), y, rows * 4, hipMemcpyDeviceToHost, st));
  DS_HIP(ctx, hipStreamSynchronize(st));
  ds_arena_reset(ctx);
  const float full = h[rows - 1];
  for (int t = 0; t < num_k; ++t) {
    fid_minus[t] = fabsf(full - h[2 * t]);
    fid_plus[t] = fabsf(full - h[2 * t + 1]);
  }
  return DS_OK;
}
