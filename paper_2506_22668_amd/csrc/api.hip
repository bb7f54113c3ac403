// C ABI entry points: argument checks, workspace, and the end-to-end explanation.
#include "internal.h"

#include <string>
#include <condition_variable>
#include <mutex>
#include <thread>

int ds_fail(ds_ctx* ctx, int code, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

int ds_arena_reserve(ds_ctx* ctx, size_t bytes) {
  if (ctx->arena_used != 0) return ds_fail(ctx, DS_EINTERNAL, "arena reserve while allocations are live");
  bytes = ds_align(bytes) + 4096;
  if (bytes <= ctx->arena_bytes) return DS_OK;
  if (ctx->arena) {
    hipStreamSynchronize(ctx->stream);
    hipFree(ctx->arena);
    ctx->arena = nullptr;
    ctx->arena_bytes = 0;
  }
  if (hipMalloc((void**)&ctx->arena, bytes) != hipSuccess) {
    (void)hipGetLastError();
    return ds_fail(ctx, DS_ENOMEM, "cannot allocate a %zu-byte workspace", bytes);
  }
  ctx->arena_bytes = bytes;
  return DS_OK;
}

void* ds_arena_alloc(ds_ctx* ctx, size_t bytes) {
  bytes = ds_align(bytes ? bytes : 1);
  if (ctx->arena_used + bytes > ctx->arena_bytes) return nullptr;
  void* p = ctx->arena + ctx->arena_used;
  ctx->arena_used += bytes;
  return p;
}

int ds_kernel_mark(ds_ctx* ctx, int slot, int end) {
  DS_HIP(ctx, hipEventRecord(ctx->kev[2 * slot + end], ctx->stream));
  if (end) ctx->kev_set[slot] = true;
  return DS_OK;
}

static void kernel_times(ds_ctx* ctx, ds_report* rep) {
  float* out[5] = {&rep->ms_k_eval, &rep->ms_k_gram, &rep->ms_k_chol, &rep->ms_k_cgls, &rep->ms_k_stream};
  for (int s = 0; s < 5; ++s) {
    *out[s] = 0.f;
    if (ctx->kev_set[s]) (void)hipEventElapsedTime(out[s], ctx->kev[2 * s], ctx->kev[2 * s + 1]);
  }
}

int ds_mail_fetch(ds_ctx* ctx, int count) {
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail, ctx->d_mail, count * sizeof(int64_t), hipMemcpyDeviceToHost, ctx->stream));
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return DS_OK;
}

extern "C" {

const char* ds_version(void) { return "distshap-hip 0.1 (gfx950)"; }

int ds_create(ds_ctx** out, int device, void* stream) {
  if (!out) return DS_EINVAL;
  *out = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return DS_EDEVICE;
  if (hipSetDevice(device) != hipSuccess) return DS_EDEVICE;
  ds_ctx* ctx = new ds_ctx();
  ctx->device = device;
  ctx->stream = (hipStream_t)stream;
  ctx->err[0] = 0;
  ctx->N = ctx->nnz = 0;
  ctx->row_ptr = nullptr;
  ctx->col = nullptr;
  ctx->X = nullptr;
  ctx->d0 = 0;
  ctx->L = 0;
  ctx->transform_dtype = DS_F32;
  ctx->model_version = 0;
  ctx->arena = nullptr;
  ctx->arena_bytes = ctx->arena_used = 0;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) { delete ctx; return DS_EDEVICE; }
  ctx->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  if (hipMalloc((void**)&ctx->d_mail, 64 * sizeof(int64_t)) != hipSuccess ||
      hipHostMalloc((void**)&ctx->h_mail, 64 * sizeof(int64_t), hipHostMallocDefault) != hipSuccess) {
    delete ctx;
    return DS_ENOMEM;
  }
  for (int i = 0; i < 6; ++i)
    if (hipEventCreate(&ctx->ev[i]) != hipSuccess) { delete ctx; return DS_EDEVICE; }
  for (int i = 0; i < 10; ++i)
    if (hipEventCreate(&ctx->kev[i]) != hipSuccess) { delete ctx; return DS_EDEVICE; }
  for (int i = 0; i < 5; ++i) ctx->kev_set[i] = false;
  ctx->owns_stream = false;
  memset(&ctx->tuning, 0, sizeof(ctx->tuning));
  ctx->cg_spare = nullptr;
  ctx->cg_spare_bytes = 0;
  ctx->h_stage = nullptr;
  ctx->h_stage_bytes = 0;
  ctx->stage_busy = false;
  if (hipEventCreate(&ctx->stage_ev) != hipSuccess) { delete ctx; return DS_EDEVICE; }
  if (hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->fork_ev, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->join_ev, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->fork2_ev, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->join2_ev, hipEventDisableTiming) != hipSuccess) { delete ctx; return DS_EDEVICE; }
  if (hipMemset(ctx->d_mail, 0, 64 * sizeof(int64_t)) != hipSuccess) { delete ctx; return DS_EDEVICE; }
  if (ds_static_scratch_init(device) != DS_OK) { delete ctx; return DS_EDEVICE; }
  *out = ctx;
  return DS_OK;
}

int ds_destroy(ds_ctx* ctx) {
  if (!ctx) return DS_OK;
  hipSetDevice(ctx->device);
  for (ds_ctx* w : ctx->workers) ds_destroy(w);
  ctx->workers.clear();
  hipStreamSynchronize(ctx->stream);
  for (ds_cgraph* g : ctx->graphs) {
    if (g->block) hipFree(g->block);
    delete g;
  }
  ctx->graphs.clear();
  if (ctx->arena) hipFree(ctx->arena);
  if (ctx->cg_spare) hipFree(ctx->cg_spare);
  if (ctx->h_stage) hipHostFree(ctx->h_stage);
  hipEventDestroy(ctx->stage_ev);
  hipStreamSynchronize(ctx->side);
  hipStreamDestroy(ctx->side);
  hipEventDestroy(ctx->fork_ev);
  hipEventDestroy(ctx->join_ev);
  hipEventDestroy(ctx->fork2_ev);
  hipEventDestroy(ctx->join2_ev);
  if (ctx->d_mail) hipFree(ctx->d_mail);
  if (ctx->h_mail) hipHostFree(ctx->h_mail);
  for (int i = 0; i < 6; ++i) hipEventDestroy(ctx->ev[i]);
  for (int i = 0; i < 10; ++i) hipEventDestroy(ctx->kev[i]);
  if (ctx->owns_stream) hipStreamDestroy(ctx->stream);
  delete ctx;
  return DS_OK;
}

const char* ds_last_error(const ds_ctx* ctx) { return ctx ? ctx->err : "null context"; }

int ds_set_graph(ds_ctx* ctx, int64_t num_nodes, const int64_t* row_ptr, const int32_t* col) {
  if (!ctx) return DS_EINVAL;
  if (num_nodes < 0 || num_nodes > 0x7fffffffLL || !row_ptr || (!col && num_nodes > 0))
    return ds_fail(ctx, DS_EINVAL, "bad graph arguments (N=%lld)", (long long)num_nodes);
  DS_HIP(ctx, hipSetDevice(ctx->device));
  ctx->N = num_nodes;
  ctx->row_ptr = row_ptr;
  ctx->col = col;
  int rc = ds_validate_csr(ctx);
  if (rc != DS_OK) {
    ctx->row_ptr = nullptr;
    ctx->col = nullptr;
    ctx->N = 0;
  }
  return rc;
}

int ds_set_tuning(ds_ctx* ctx, const ds_tuning* tuning) {
  if (!ctx) return DS_EINVAL;
  if (!tuning) {
    memset(&ctx->tuning, 0, sizeof(ctx->tuning));
    return DS_OK;
  }
  if (tuning->batch_workers < 0 || tuning->batch_workers > 16 || tuning->gram_sparse_div < 0 ||
      !(tuning->gram_dense_fraction >= 0.f && tuning->gram_dense_fraction <= 1.f) || tuning->sampler_window < -1 ||
      tuning->eval_path < 0 || tuning->eval_path > 4 ||
      (tuning->cgls_dense_div != 0 && (tuning->cgls_dense_div < 32 || tuning->cgls_dense_div > 65536)) ||
      tuning->pair_lists < -1 || (tuning->pair_lists > 0 && (tuning->pair_lists < 16 || tuning->pair_lists > (1 << 20))))
    return ds_fail(ctx, DS_EINVAL, "tuning value out of range");
  ctx->tuning = *tuning;
  return DS_OK;
}

int ds_set_features(ds_ctx* ctx, const void* X, int32_t d0, int32_t dtype) {
  if (!ctx) return DS_EINVAL;
  if (!X || d0 < 1 || dtype != DS_F32) return ds_fail(ctx, DS_EINVAL, "features must be fp32 with d0 >= 1");
  ctx->X = (const float*)X;
  ctx->d0 = d0;
  return DS_OK;
}

int ds_set_gcn(ds_ctx* ctx, int32_t num_layers, const int32_t* dims, const void* const* W, const void* const* bias,
               int32_t transform_dtype) {
  if (!ctx) return DS_EINVAL;
  if (num_layers < 1 || num_layers > DS_MAX_LAYERS || !dims || !W)
    return ds_fail(ctx, DS_EINVAL, "the GCN needs 1..%d layers", DS_MAX_LAYERS);
  if (transform_dtype != DS_F32 && transform_dtype != DS_BF16_IN_F32_ACC)
    return ds_fail(ctx, DS_EINVAL, "unknown transform dtype %d", transform_dtype);
  for (int l = 0; l <= num_layers; ++l)
    if (dims[l] < 1 || dims[l] > 4096) return ds_fail(ctx, DS_EINVAL, "layer width %d out of range [1, 4096]", dims[l]);
  if (dims[num_layers] > 1024) return ds_fail(ctx, DS_EINVAL, "at most 1024 classes");
  for (int l = 0; l < num_layers; ++l)
    if (!W[l]) return ds_fail(ctx, DS_EINVAL, "weight matrix %d is null", l);
  ctx->L = num_layers;
  for (int l = 0; l <= num_layers; ++l) ctx->dims[l] = dims[l];
  for (int l = 0; l < num_layers; ++l) {
    ctx->W[l] = (const float*)W[l];
    ctx->bias[l] = bias ? (const float*)bias[l] : nullptr;
  }
  ctx->transform_dtype = transform_dtype;
  ctx->model_kind = DS_MODEL_GCN;
  ctx->model_version += 1;
  return DS_OK;
}

int ds_set_gat(ds_ctx* ctx, int32_t num_layers, const int32_t* head_dims, const int32_t* heads, const void* const* W,
               const void* const* att_src, const void* const* att_dst, const void* const* bias, float negative_slope) {
  if (!ctx) return DS_EINVAL;
  if (num_layers < 1 || num_layers > DS_MAX_LAYERS || !head_dims || !heads || !W || !att_src || !att_dst)
    return ds_fail(ctx, DS_EINVAL, "the GAT needs 1..%d layers with weights and attention vectors", DS_MAX_LAYERS);
  if (head_dims[0] < 1 || head_dims[0] > 4096) return ds_fail(ctx, DS_EINVAL, "input width %d out of range [1, 4096]", head_dims[0]);
  for (int l = 0; l < num_layers; ++l) {
    if (heads[l] < 1 || heads[l] > 64) return ds_fail(ctx, DS_EINVAL, "layer %d: %d heads out of range [1, 64]", l + 1, heads[l]);
    if (head_dims[l + 1] < 1 || (int64_t)heads[l] * head_dims[l + 1] > 4096)
      return ds_fail(ctx, DS_EINVAL, "layer %d: transform width %lld out of range [1, 4096]", l + 1, (long long)heads[l] * head_dims[l + 1]);
    if (!W[l] || !att_src[l] || !att_dst[l]) return ds_fail(ctx, DS_EINVAL, "layer %d: null weight or attention pointer", l + 1);
  }
  if (head_dims[num_layers] > 1024) return ds_fail(ctx, DS_EINVAL, "at most 1024 classes");
  if (!(negative_slope >= 0.f && negative_slope <= 1.f)) return ds_fail(ctx, DS_EINVAL, "negative_slope must lie in [0, 1]");
  ctx->L = num_layers;
  ctx->dims[0] = head_dims[0];
  for (int l = 0; l < num_layers; ++l) {
    ctx->gat.heads[l] = heads[l];
    ctx->gat.fh[l] = head_dims[l + 1];
    ctx->gat.zw[l] = heads[l] * head_dims[l + 1];
    ctx->dims[l + 1] = l + 1 < num_layers ? ctx->gat.zw[l] : head_dims[l + 1];
    ctx->W[l] = (const float*)W[l];
    ctx->gat.att_src[l] = (const float*)att_src[l];
    ctx->gat.att_dst[l] = (const float*)att_dst[l];
    ctx->bias[l] = bias ? (const float*)bias[l] : nullptr;
  }
  ctx->gat.slope = negative_slope;
  ctx->transform_dtype = DS_F32;
  ctx->model_kind = DS_MODEL_GAT;
  ctx->model_version += 1;
  return DS_OK;
}

static ds_options default_options(const ds_options* in) {
  ds_options o;
  memset(&o, 0, sizeof(o));
  if (in) o = *in;
  return o;
}

int ds_extract(ds_ctx* ctx, int64_t target, const ds_options* opts, ds_cgraph** out) {
  if (!ctx || !out) return DS_EINVAL;
  *out = nullptr;
  DS_HIP(ctx, hipSetDevice(ctx->device));
  ds_options o = default_options(opts);
  int hops = o.hops > 0 ? o.hops : ctx->L;
  if (hops < 1) return ds_fail(ctx, DS_EINVAL, "hops is 0 and no model is set");
  if (ctx->d0 > 0 && ctx->L > 0 && ctx->d0 != ctx->dims[0])
    return ds_fail(ctx, DS_EINVAL, "feature width %d does not match the model's input width %d", ctx->d0, ctx->dims[0]);
  return ds_extract_impl(ctx, target, hops, o.directed ? 1 : 0, out);
}

int ds_cgraph_get_info(const ds_cgraph* cg, ds_cgraph_info* info) {
  if (!cg || !info) return DS_EINVAL;
  *info = cg->info;
  return DS_OK;
}

// local ids -> global ids for the player list
__global__ void export_edges_kernel(const int2* pl, const int64_t* node_gid, int64_t n,
                                    int64_t* es, int64_t* ed) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= n) return;
  const int2 e = pl[p];
  if (es) es[p] = node_gid[e.x];
  if (ed) ed[p] = node_gid[e.y];
}

int ds_cgraph_edges(ds_ctx* ctx, const ds_cgraph* cg, int64_t* edge_src, int64_t* edge_dst) {
  if (!ctx || !cg) return DS_EINVAL;
  const int64_t n = cg->info.num_players;
  if (n == 0 || (!edge_src && !edge_dst)) return DS_OK;
  hipLaunchKernelGGL(export_edges_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, cg->pl,
                     cg->node_gid, n, edge_src, edge_dst);
  DS_HIP(ctx, hipGetLastError());
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return DS_OK;
}

int ds_cgraph_nodes(ds_ctx* ctx, const ds_cgraph* cg, int64_t* node_gid, int32_t* hop) {
  if (!ctx || !cg) return DS_EINVAL;
  const int64_t V = cg->info.num_nodes;
  if (node_gid) DS_HIP(ctx, hipMemcpyAsync(node_gid, cg->node_gid, V * 8, hipMemcpyDeviceToDevice, ctx->stream));
  if (hop) DS_HIP(ctx, hipMemcpyAsync(hop, cg->hop, V * 4, hipMemcpyDeviceToDevice, ctx->stream));
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return DS_OK;
}

int ds_cgraph_first_transform(ds_ctx* ctx, ds_cgraph* cg, float* out) {
  if (!ctx || !cg || !out) return DS_EINVAL;
  ds_arena_reset(ctx);
  DS_TRY(ds_arena_reserve(ctx, ds_eval_arena_bytes(ctx, cg, 1)));
  int rc = ds_prepare_model(ctx, cg);
  ds_arena_reset(ctx);
  DS_TRY(rc);
  DS_HIP(ctx, hipMemcpyAsync(out, cg->P, (size_t)cg->info.num_nodes * ds_first_width(ctx) * 4, hipMemcpyDeviceToDevice, ctx->stream));
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return DS_OK;
}

int ds_cgraph_free(ds_ctx* ctx, ds_cgraph* cg) {
  if (!cg) return DS_OK;
  if (!ctx) ctx = cg->owner;
  for (size_t i = 0; i < ctx->graphs.size(); ++i)
    if (ctx->graphs[i] == cg) {
      ctx->graphs.erase(ctx->graphs.begin() + i);
      break;
    }
  if (cg->block) {
    // keep the larger of (this block, the spare) for the next extraction; later work on the
    // context's stream is ordered after everything that still reads the block
    if (cg->block_bytes > ctx->cg_spare_bytes) {
      if (ctx->cg_spare) {
        hipStreamSynchronize(ctx->stream);
        hipFree(ctx->cg_spare);
      }
      ctx->cg_spare = cg->block;
      ctx->cg_spare_bytes = cg->block_bytes;
    } else {
      hipStreamSynchronize(ctx->stream);
      hipFree(cg->block);
    }
  }
  delete cg;
  return DS_OK;
}

static int sample_checked(ds_ctx* ctx, int64_t n, int64_t n_samples, uint64_t seed, uint32_t tag, int64_t pb, int64_t pe,
                          bool whole, uint64_t* Z, float* w, int32_t* sz, int64_t* k_out, const ds_options* opts = nullptr) {
  if (!ctx) return DS_EINVAL;
  if (!Z || !w || !sz) return ds_fail(ctx, DS_EINVAL, "null output buffer");
  DS_HIP(ctx, hipSetDevice(ctx->device));
  ds_plan plan;
  DS_TRY(ds_make_plan(ctx, n, n_samples, &plan, opts ? opts->weighting : DS_WEIGHT_CLASS_MASS, opts ? opts->saturate : 0));
  if (whole) { pb = 0; pe = plan.k / 2; }
  ds_arena_reset(ctx);
  DS_TRY(ds_arena_reserve(ctx, ds_sample_arena_bytes(plan)));
  int rc = ds_sample_launch(ctx, plan, seed, tag, pb, pe, Z, w, sz);
  if (rc == DS_OK) rc = ds_sample_check(ctx);
  ds_arena_reset(ctx);
  if (k_out) *k_out = plan.k;
  return rc;
}

int ds_sample(ds_ctx* ctx, int64_t n, int64_t n_samples, uint64_t seed, uint32_t tag, uint64_t* Z, float* w,
              int32_t* sz, int64_t* k_out) {
  return sample_checked(ctx, n, n_samples, seed, tag, 0, 0, true, Z, w, sz, k_out);
}

int ds_sample_ex(ds_ctx* ctx, int64_t n, int64_t n_samples, uint64_t seed, uint32_t tag, const ds_options* opts, uint64_t* Z,
                 float* w, int32_t* sz, int64_t* k_out) {
  if (ctx && opts && opts->weighting != DS_WEIGHT_CLASS_MASS && opts->weighting != DS_WEIGHT_UNIFORM)
    return ds_fail(ctx, DS_EINVAL, "unknown weighting %d", opts->weighting);
  return sample_checked(ctx, n, n_samples, seed, tag, 0, 0, true, Z, w, sz, k_out, opts);
}

int ds_sample_range(ds_ctx* ctx, int64_t n, int64_t n_samples, uint64_t seed, uint32_t tag, int64_t pair_begin,
                    int64_t pair_end, uint64_t* Z, float* w, int32_t* sz) {
  return sample_checked(ctx, n, n_samples, seed, tag, pair_begin, pair_end, false, Z, w, sz, nullptr);
}

static int eval_checked(ds_ctx* ctx, const ds_cgraph* cg_in, const uint64_t* Z, int64_t k, int32_t score, float* y,
                        int32_t* pred_class_out, int flags);

int ds_eval(ds_ctx* ctx, const ds_cgraph* cg_in, const uint64_t* Z, int64_t k, int32_t score, float* y,
            int32_t* pred_class_out) {
  return eval_checked(ctx, cg_in, Z, k, score, y, pred_class_out, 0);
}

int ds_eval_pairs(ds_ctx* ctx, const ds_cgraph* cg_in, const uint64_t* Z, int64_t k, int32_t score, float* y,
                  int32_t* pred_class_out) {
  if (ctx && (k & 1)) return ds_fail(ctx, DS_EINVAL, "ds_eval_pairs needs an even number of rows (k=%lld)", (long long)k);
  return eval_checked(ctx, cg_in, Z, k, score, y, pred_class_out, DS_EVAL_PAIRED);
}

static int eval_checked(ds_ctx* ctx, const ds_cgraph* cg_in, const uint64_t* Z, int64_t k, int32_t score, float* y,
                        int32_t* pred_class_out, int flags) {
  if (!ctx || !cg_in) return DS_EINVAL;
  if (k < 0 || (k > 0 && (!Z || !y))) return ds_fail(ctx, DS_EINVAL, "bad eval arguments");
  if (score != DS_SCORE_PROB && score != DS_SCORE_LOGIT) return ds_fail(ctx, DS_EINVAL, "unknown score %d", score);
  DS_HIP(ctx, hipSetDevice(ctx->device));
  ds_cgraph* cg = const_cast<ds_cgraph*>(cg_in);
  ds_arena_reset(ctx);
  DS_TRY(ds_arena_reserve(ctx, ds_eval_arena_bytes(ctx, cg, k)));
  for (int i = 0; i < 5; ++i) ctx->kev_set[i] = false;
  int rc = ds_eval_impl(ctx, cg, Z, k, score, y, flags);
  if (rc == DS_OK && hipStreamSynchronize(ctx->stream) != hipSuccess) rc = ds_fail(ctx, DS_EDEVICE, "eval kernel failed");
  ds_arena_reset(ctx);
  if (rc == DS_OK && pred_class_out) {
    rc = ds_fetch_pred_class(ctx, cg);
    *pred_class_out = cg->pred_class;
  }
  return rc;
}

int ds_eval_noalloc(ds_ctx* ctx, const ds_cgraph* cg_in, const uint64_t* Z, int64_t k, int32_t score, float* y) {
  if (!ctx || !cg_in) return DS_EINVAL;
  if (k < 0 || (k > 0 && (!Z || !y))) return ds_fail(ctx, DS_EINVAL, "bad eval arguments");
  if (score != DS_SCORE_PROB && score != DS_SCORE_LOGIT) return ds_fail(ctx, DS_EINVAL, "unknown score %d", score);
  if (ctx->model_kind != DS_MODEL_GCN) return ds_fail(ctx, DS_EINVAL, "ds_eval_noalloc covers the GCN only");
  DS_HIP(ctx, hipSetDevice(ctx->device));
  void* ptr = ds_static_scratch(ctx->device);
  if (!ptr) return ds_fail(ctx, DS_EINTERNAL, "the static scratch array of device %d was not initialised", ctx->device);
  ds_cgraph* cg = const_cast<ds_cgraph*>(cg_in);
  // the same host driver and kernels as ds_eval, with the workspace pointed at the static array for this call
  char* const own = ctx->arena;
  const size_t own_bytes = ctx->arena_bytes, own_used = ctx->arena_used;
  ctx->arena = (char*)ptr;
  ctx->arena_bytes = DS_EVAL_NOALLOC_SCRATCH_BYTES;
  ctx->arena_used = 0;
  int rc = DS_OK;
  const size_t W = (size_t)((cg->info.num_players + 63) / 64);
  const size_t fixed = ds_align(W * 8 + 8) + ds_align((size_t)ctx->dims[ctx->L] * 4 + 8) + 4096;
  if (fixed > DS_EVAL_NOALLOC_SCRATCH_BYTES)
    rc = ds_fail(ctx, DS_ECAPACITY, "ds_eval_noalloc: %lld players need %zu bytes of scratch, the static array holds %u",
                 (long long)cg->info.num_players, fixed, DS_EVAL_NOALLOC_SCRATCH_BYTES);
  if (rc == DS_OK) rc = ds_eval_impl(ctx, cg, Z, k, score, y, DS_EVAL_BOUNDED);
  if (rc == DS_EINTERNAL) rc = DS_ECAPACITY;  // the bounded workspace ran out: a size limit, not a fault
  ctx->arena = own;
  ctx->arena_bytes = own_bytes;
  ctx->arena_used = own_used;
  return rc;
}

static int solve_dispatch(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, const float* y,
                          const ds_options& o, int paired, float* phi, ds_report* rep) {
  int solver = o.solver;
  if (solver == DS_SOLVER_AUTO) solver = n <= 16384 ? DS_SOLVER_GRAM_CHOL : DS_SOLVER_CGLS;
  int rc = DS_OK;
  if (solver == DS_SOLVER_GRAM_CHOL) {
    rc = ds_solve_gram_chol(ctx, n, k, Z, w, y, paired, phi);
    if (rc == DS_ESINGULAR && o.solver == DS_SOLVER_AUTO) solver = DS_SOLVER_CGLS;  // fall through to the minimum-norm solve
  }
  int iters = 0;
  double rel = 0.0;
  if (solver == DS_SOLVER_CGLS) rc = ds_solve_cgls_impl(ctx, n, k, Z, w, y, paired, o.tol, o.max_iter, phi, &iters, &rel);
  if (rep) {
    rep->solver_used = solver;
    rep->cgls_iterations = iters;
    rep->cgls_rel_residual = rel;
  }
  return rc;
}

static size_t solve_arena_bytes(int64_t n, int64_t k, int solver_opt) {
  size_t a = 0, b = 0;
  if (solver_opt != DS_SOLVER_CGLS && (solver_opt == DS_SOLVER_GRAM_CHOL || n <= 16384)) a = ds_gram_arena_bytes(n, k);
  if (solver_opt != DS_SOLVER_GRAM_CHOL) b = ds_cgls_arena_bytes(n, k);
  if (solver_opt == DS_SOLVER_AUTO && n > 16384) a = 0;
  return a > b ? a : b;
}

int ds_solve(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, const float* y,
             const ds_options* opts, float* phi, ds_report* report) {
  if (!ctx) return DS_EINVAL;
  if (n < 2 || k < 2 || !Z || !w || !y || !phi) return ds_fail(ctx, DS_EINVAL, "bad solve arguments (n=%lld, k=%lld)", (long long)n, (long long)k);
  DS_HIP(ctx, hipSetDevice(ctx->device));
  ds_options o = default_options(opts);
  if (report) memset(report, 0, sizeof(*report));
  ds_arena_reset(ctx);
  DS_TRY(ds_arena_reserve(ctx, solve_arena_bytes(n, k, o.solver)));
  for (int i = 0; i < 5; ++i) ctx->kev_set[i] = false;
  int rc = solve_dispatch(ctx, n, k, Z, w, y, o, o.paired ? 1 : 0, phi, report);
  hipStreamSynchronize(ctx->stream);
  ds_arena_reset(ctx);
  if (report) {
    kernel_times(ctx, report);
    report->num_players = n;
    report->num_rows = k;
  }
  return rc;
}

__global__ void single_player_kernel(const float* y, float* phi) { phi[0] = y[1] - y[0]; }

__global__ void copy_probe_kernel(uint4* dst, const uint4* src, int64_t count) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

int ds_copy_probe(ds_ctx* ctx, void* dst, const void* src, int64_t bytes) {
  if (!ctx || !dst || !src || bytes < 0 || (bytes & 15)) return ds_fail(ctx, DS_EINVAL, "copy probe: bytes must be a non-negative multiple of 16");
  if (bytes == 0) return DS_OK;
  hipLaunchKernelGGL(copy_probe_kernel, dim3(ctx->num_cus * 16), dim3(256), 0, ctx->stream, (uint4*)dst, (const uint4*)src, bytes / 16);
  DS_HIP(ctx, hipGetLastError());
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  return DS_OK;
}

static int explain_extracted(ds_ctx* ctx, ds_cgraph* cg, int64_t target, int64_t n_samples, uint64_t seed, const ds_options& o,
                             float* phi, int64_t* M_inout, int64_t* edge_src, int64_t* edge_dst, ds_report* report);

// what ds_explain reads back at its end, in mailbox slots out[0..4]: (y[0], y[1]) as two floats | unused | predicted
// class | sampler overflow flag | pivot flag of the factorisation (0 without one)
__global__ void final_mail_kernel(const float* y, const int32_t* pred, const int64_t* sampler_flag, const int* pivot_flag,
                                  int64_t* out) {
  float* f = (float*)out;
  f[0] = y[0];
  f[1] = y[1];
  out[1] = 0;
  out[2] = (int64_t)*pred;
  out[3] = *sampler_flag;
  out[4] = pivot_flag ? (int64_t)*pivot_flag : 0;
}

int ds_explain(ds_ctx* ctx, int64_t target, int64_t n_samples, uint64_t seed, const ds_options* opts, float* phi,
               int64_t* M_inout, int64_t* edge_src, int64_t* edge_dst, ds_report* report) {
  if (!ctx || !M_inout) return DS_EINVAL;
  DS_HIP(ctx, hipSetDevice(ctx->device));
  ds_options o = default_options(opts);
  hipStream_t st = ctx->stream;
  if (ctx->L < 1) return ds_fail(ctx, DS_EINVAL, "no model is set (ds_set_gcn / ds_set_gat)");
  for (int i = 0; i < 5; ++i) ctx->kev_set[i] = false;
  DS_HIP(ctx, hipEventRecord(ctx->ev[0], st));
  ds_cgraph* cg = nullptr;
  DS_TRY(ds_extract(ctx, target, &o, &cg));
  return explain_extracted(ctx, cg, target, n_samples, seed, o, phi, M_inout, edge_src, edge_dst, report);
}

// Everything after the extraction; takes over (and frees) the computational graph. ctx->ev[0] has been recorded
// before the extraction.
static int explain_extracted(ds_ctx* ctx, ds_cgraph* cg, int64_t target, int64_t n_samples, uint64_t seed, const ds_options& o,
                             float* phi, int64_t* M_inout, int64_t* edge_src, int64_t* edge_dst, ds_report* report) {
  ds_report rep;
  memset(&rep, 0, sizeof(rep));
  hipStream_t st = ctx->stream;
  struct Guard {
    ds_ctx* c; ds_cgraph* g;
    ~Guard() { (void)hipStreamSynchronize(c->side); c->lists = ds_pair_lists{}; ds_cgraph_free(c, g); ds_arena_reset(c); }
  } guard{ctx, cg};
  const int64_t n = cg->info.num_players;
  rep.num_players = n;
  rep.num_nodes = cg->info.num_nodes;
  rep.num_entries = cg->info.num_entries;
  const int64_t capacity = *M_inout;
  *M_inout = n;
  if (n > capacity) return ds_fail(ctx, DS_ECAPACITY, "phi holds %lld entries but the computational graph has %lld players", (long long)capacity, (long long)n);
  if (n > 0 && !phi) return ds_fail(ctx, DS_EINVAL, "phi is null");
  if (n == 0) {
    if (report) *report = rep;
    return DS_OK;
  }
  DS_TRY(ds_cgraph_edges(ctx, cg, edge_src, edge_dst));
  DS_HIP(ctx, hipEventRecord(ctx->ev[1], st));

  const int64_t W = (n + 63) / 64;
  int64_t k;
  ds_plan plan;
  if (n == 1) {
    k = 2;
  } else {
    if (o.weighting != DS_WEIGHT_CLASS_MASS && o.weighting != DS_WEIGHT_UNIFORM)
      return ds_fail(ctx, DS_EINVAL, "unknown weighting %d", o.weighting);
    DS_TRY(ds_make_plan(ctx, n, n_samples, &plan, o.weighting, o.saturate ? 1 : 0));
    k = plan.k;
  }
  rep.num_rows = k;
  rep.enumerated = n >= 2 ? plan.enumerate : 1;
  // workspace: Z, w, sz, y live for the whole call; stage temporaries follow them
  size_t persistent = ds_align((size_t)k * W * 8) + ds_align(k * 4) * 3 + 1024 + ds_eval_arena_bytes(ctx, cg, 1);
  size_t stage = n >= 2 ? ds_sample_arena_bytes(plan) : 0;
  size_t e = ds_eval_arena_bytes(ctx, cg, k);
  if (e > stage) stage = e;
  if (n >= 2) {
    size_t s = solve_arena_bytes(n, k, o.solver);
    if (s > stage) stage = s;
    // the direct solver's buffers are live during the inference, and a fall-back CGLS comes on top of them
    if (o.solver == DS_SOLVER_GRAM_CHOL || (o.solver == DS_SOLVER_AUTO && n <= 16384)) persistent += ds_gram_arena_bytes(n, k);
  }
  // Long mask rows: the inference reads the sparse small members (at most n / 64 players: a list is then at most half
  // the bytes of the bit row) as player lists that the sampler writes beside the rows, instead of streaming their bits.
  ds_pair_lists lists{};
  if (n >= 2 && ctx->tuning.pair_lists != -1 && ds_sampler_lists_possible(ctx, plan) && ds_eval_streams_pairs(ctx, cg, k)) {
    const int64_t div = ctx->tuning.pair_lists > 0 ? ctx->tuning.pair_lists : 64;
    lists.max_size = n / div < plan.H ? n / div : plan.H;
    lists.total = ds_pair_list_entries(plan, lists.max_size);
    if (lists.total > 0) persistent += ds_align((size_t)lists.total * 4) + ds_align((size_t)(k / 2) * 8);
  }
  ds_arena_reset(ctx);
  DS_TRY(ds_arena_reserve(ctx, persistent + stage));
  uint64_t* Z = (uint64_t*)ds_arena_alloc(ctx, (size_t)k * W * 8);
  float* w = (float*)ds_arena_alloc(ctx, k * 4);
  int32_t* sz = (int32_t*)ds_arena_alloc(ctx, k * 4);
  float* y = (float*)ds_arena_alloc(ctx, k * 4);
  if (!Z || !w || !sz || !y) return ds_fail(ctx, DS_EINTERNAL, "explain: arena exhausted");
  if (lists.total > 0) {
    lists.entries = (uint32_t*)ds_arena_alloc(ctx, (size_t)lists.total * 4);
    lists.offset = (int64_t*)ds_arena_alloc(ctx, (size_t)(k / 2) * 8);
    if (!lists.entries || !lists.offset) return ds_fail(ctx, DS_EINTERNAL, "explain: arena exhausted");
  }
  // The shared first transform and the predicted class depend only on the computational graph:
  // they run on the side stream while the main stream draws the coalitions.
  DS_HIP(ctx, hipEventRecord(ctx->fork_ev, st));
  DS_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->fork_ev, 0));
  {
    ctx->stream = ctx->side;
    const int prc = ds_prepare_model(ctx, cg);  // its temporaries stay allocated below `mark`
    ctx->stream = st;
    DS_TRY(prc);
    DS_HIP(ctx, hipEventRecord(ctx->join_ev, ctx->side));
  }
  const size_t mark = ctx->arena_used;

  if (n == 1) {
    const uint64_t rows[2] = {0ull, 1ull};
    DS_HIP(ctx, hipMemcpyAsync(Z, rows, sizeof(rows), hipMemcpyHostToDevice, st));
    DS_HIP(ctx, hipStreamSynchronize(st));
  } else {
    DS_TRY(ds_sample_launch(ctx, plan, seed, (uint32_t)((uint64_t)target & 0xFFFFFFFFull), 0, k / 2, Z, w, sz,
                            lists.entries ? &lists : nullptr));
  }
  ctx->arena_used = mark;
  DS_HIP(ctx, hipEventRecord(ctx->ev[2], st));

  // The Gram matrix and the system matrix of the direct solver need the masks and weights but not
  // the model outputs: they are built on the side stream while the main stream runs the inference.
  const bool direct = n >= 2 && (o.solver == DS_SOLVER_GRAM_CHOL || (o.solver == DS_SOLVER_AUTO && n <= 16384));
  ds_gram_state gs;
  if (direct) {
    DS_HIP(ctx, hipEventRecord(ctx->fork2_ev, st));
    DS_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->fork2_ev, 0));
    ctx->stream = ctx->side;
    const int grc = ds_gram_begin(ctx, n, k, Z, w, 1, &gs);  // its buffers stay allocated below `mark2`
    ctx->stream = st;
    DS_TRY(grc);
    DS_HIP(ctx, hipEventRecord(ctx->join2_ev, ctx->side));
  }
  const size_t mark2 = ctx->arena_used;

  DS_HIP(ctx, hipStreamWaitEvent(st, ctx->join_ev, 0));
  ctx->lists = lists;
  const int erc = ds_eval_impl(ctx, cg, Z, k, o.score, y, DS_EVAL_PAIRED, n >= 2 ? sz : nullptr);  // the sampler's rows are complementary pairs
  ctx->lists = ds_pair_lists{};
  DS_TRY(erc);
  ctx->arena_used = mark2;
  DS_HIP(ctx, hipEventRecord(ctx->ev[3], st));

  int rc = DS_OK;
  if (n == 1) {
    hipLaunchKernelGGL(single_player_kernel, dim3(1), dim3(1), 0, st, y, phi);
  } else if (direct) {
    DS_HIP(ctx, hipStreamWaitEvent(st, ctx->join2_ev, 0));
    rc = ds_gram_finish(ctx, &gs, Z, w, y, phi, 1);  // the pivot flag comes back with the final read-back
    rep.solver_used = DS_SOLVER_GRAM_CHOL;
  } else {
    rc = solve_dispatch(ctx, n, k, Z, w, y, o, 1, phi, &rep);
  }
  if (rc != DS_OK && rc != DS_ENOTCONV) return rc;
  DS_HIP(ctx, hipEventRecord(ctx->ev[4], st));
  // one round trip for everything the host still needs: f(empty), f(full), predicted class, sampler flag, pivot
  // flag, gathered into consecutive mailbox slots by one small kernel and copied once
  float* f01 = (float*)(ctx->h_mail + 32);
  hipLaunchKernelGGL(final_mail_kernel, dim3(1), dim3(1), 0, st, y, cg->d_pred, ctx->d_mail + DS_MAIL_SAMPLER,
                     direct ? gs.flag : (const int*)nullptr, ctx->d_mail + 32);
  DS_HIP(ctx, hipGetLastError());
  DS_HIP(ctx, hipMemcpyAsync(ctx->h_mail + 32, ctx->d_mail + 32, 5 * sizeof(int64_t), hipMemcpyDeviceToHost, st));
  DS_HIP(ctx, hipStreamSynchronize(st));
  if (n >= 2 && ctx->h_mail[35] != 0)
    return ds_fail(ctx, DS_EINTERNAL, "sampler: candidate list overflow (too many keys share a 24-bit prefix)");
  if (direct && *(int*)(ctx->h_mail + 36) != 0) {
    if (o.solver != DS_SOLVER_AUTO)
      return ds_fail(ctx, DS_ESINGULAR, "Cholesky met a non-positive pivot: the sampled rows do not determine all %lld players", (long long)n);
    // rank-deficient: the minimum-norm solve instead
    int iters = 0;
    double rel = 0.0;
    rc = ds_solve_cgls_impl(ctx, n, k, Z, w, y, 1, o.tol, o.max_iter, phi, &iters, &rel);
    rep.solver_used = DS_SOLVER_CGLS;
    rep.cgls_iterations = iters;
    rep.cgls_rel_residual = rel;
    if (rc != DS_OK && rc != DS_ENOTCONV) return rc;
    DS_HIP(ctx, hipEventRecord(ctx->ev[4], st));
    DS_HIP(ctx, hipStreamSynchronize(st));
  }
  rep.f_empty = f01[0];
  rep.f_full = f01[1];
  rep.pred_class = *(int32_t*)(ctx->h_mail + 34);
  cg->pred_class = rep.pred_class;
  hipEventElapsedTime(&rep.ms_extract, ctx->ev[0], ctx->ev[1]);
  hipEventElapsedTime(&rep.ms_sample, ctx->ev[1], ctx->ev[2]);
  hipEventElapsedTime(&rep.ms_eval, ctx->ev[2], ctx->ev[3]);
  hipEventElapsedTime(&rep.ms_solve, ctx->ev[3], ctx->ev[4]);
  hipEventElapsedTime(&rep.ms_total, ctx->ev[0], ctx->ev[4]);
  kernel_times(ctx, &rep);
  rep.num_pairs = k / 2 - 1;
  {
    const double row_bytes = (double)W * 8.0, half = (double)(k / 2);
    rep.bytes_sample = (double)k * row_bytes + (double)k * 8.0;
    rep.bytes_eval = half * row_bytes + (double)k * 4.0;
    rep.bytes_solve = rep.solver_used == DS_SOLVER_CGLS ? (double)rep.cgls_iterations * ctx->cgls_bytes_per_iter
                                                        : half * row_bytes + (double)n * (double)n * 4.0;
  }
  if (report) *report = rep;
  return rc;
}

// worker contexts of a batch: same graph, features and model as the parent, own stream and workspace
static int batch_workers(const ds_ctx* ctx) {
  const int x = ctx->tuning.batch_workers > 0 ? ctx->tuning.batch_workers : 8;
  return x > 16 ? 16 : x;
}

static int ensure_workers(ds_ctx* ctx, int count) {
  while ((int)ctx->workers.size() < count) {
    hipStream_t st;
    DS_HIP(ctx, hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    ds_ctx* w = nullptr;
    if (ds_create(&w, ctx->device, (void*)st) != DS_OK) {
      (void)hipStreamDestroy(st);
      return ds_fail(ctx, DS_EDEVICE, "cannot create a worker context");
    }
    w->owns_stream = true;
    ctx->workers.push_back(w);
  }
  for (ds_ctx* w : ctx->workers) {
    w->N = ctx->N; w->nnz = ctx->nnz; w->row_ptr = ctx->row_ptr; w->col = ctx->col;
    w->X = ctx->X; w->d0 = ctx->d0;
    w->L = ctx->L;
    for (int l = 0; l <= DS_MAX_LAYERS; ++l) w->dims[l] = ctx->dims[l];
    for (int l = 0; l < DS_MAX_LAYERS; ++l) { w->W[l] = ctx->W[l]; w->bias[l] = ctx->bias[l]; }
    w->transform_dtype = ctx->transform_dtype;
    w->model_version = ctx->model_version;
    w->model_kind = ctx->model_kind;
    w->gat = ctx->gat;
    w->tuning = ctx->tuning;
  }
  return DS_OK;
}

int ds_explain_batch(ds_ctx* ctx, const int64_t* targets, int32_t num_targets, int64_t n_samples, uint64_t seed,
                     const ds_options* opts, float* phi_concat, int64_t* M_out, int64_t* offsets, int64_t* edge_src,
                     int64_t* edge_dst, int64_t capacity, ds_report* reports) {
  if (!ctx || !targets || num_targets < 0 || !M_out || !offsets) return DS_EINVAL;
  DS_HIP(ctx, hipSetDevice(ctx->device));
  offsets[0] = 0;
  if (num_targets == 0) return DS_OK;
  // Several explanations (eight unless the knob says otherwise) are in flight at a time, each on its own worker
  // context and host thread: a single explanation leaves much of the GPU idle in its latency-bound stages.
  // (Measured on 1,010-player games: 1.53 / 1.21 / 1.00 / 0.96 ms per explanation with 1 / 2 / 4 / 8 in flight; the
  // launches of all workers go through one runtime, which is what the curve runs into.)
  // A target's place in the outputs depends on the sizes of all targets before it. Every worker extracts its
  // target's computational graph, publishes the size, waits until the sizes before it are known (their workers
  // publish right after their own extraction, so the wait is short and the lowest unpublished target never waits)
  // and goes on with the graph it already holds.
  if (ctx->L < 1) return ds_fail(ctx, DS_EINVAL, "no model is set (ds_set_gcn / ds_set_gat)");
  int nw = num_targets < batch_workers(ctx) ? num_targets : batch_workers(ctx);
  DS_TRY(ensure_workers(ctx, nw));
  DS_HIP(ctx, hipStreamSynchronize(ctx->stream));  // whatever the caller queued before is visible to the workers
  const ds_options o = default_options(opts);
  std::vector<int> status(num_targets, DS_OK);
  std::vector<std::string> errs(num_targets);
  // The first graph is extracted up front: large games fill the GPU on their own (and their workspaces are large),
  // so fewer of them are taken at a time, and the first target's size stands for the batch.
  ds_cgraph* first_cg = nullptr;
  {
    ds_ctx* w0 = ctx->workers[0];
    for (int i = 0; i < 5; ++i) w0->kev_set[i] = false;
    DS_HIP(ctx, hipEventRecord(w0->ev[0], w0->stream));
    const int rc = ds_extract(w0, targets[0], &o, &first_cg);
    if (rc != DS_OK) {
      strncpy(ctx->err, w0->err, sizeof(ctx->err) - 1);
      return rc;
    }
    const int64_t m0 = first_cg->info.num_players;
    if (m0 > 16384) nw = 1;
    else if (m0 > 4096 && nw > 2) nw = 2;
  }
  std::mutex mu;
  std::condition_variable cv;
  std::vector<char> published(num_targets, 0);
  int32_t prefix = 0;  // offsets[0 .. prefix] are final
  {
    std::vector<std::thread> pool;
    for (int wi = 0; wi < nw; ++wi)
      pool.emplace_back([&, wi]() {
        ds_ctx* w = ctx->workers[wi];
        (void)hipSetDevice(w->device);
        for (int32_t t = wi; t < num_targets; t += nw) {
          ds_cgraph* cg = nullptr;
          int rc = DS_OK;
          if (t == 0) {
            cg = first_cg;
          } else {
            for (int i = 0; i < 5; ++i) w->kev_set[i] = false;
            rc = hipEventRecord(w->ev[0], w->stream) == hipSuccess ? DS_OK : DS_EDEVICE;
            if (rc == DS_OK) rc = ds_extract(w, targets[t], &o, &cg);
          }
          status[t] = rc;
          if (rc != DS_OK) errs[t] = w->err;
          M_out[t] = rc == DS_OK ? cg->info.num_players : 0;
          {
            std::unique_lock<std::mutex> lk(mu);
            published[t] = 1;
            while (prefix < num_targets && published[prefix]) {
              offsets[prefix + 1] = offsets[prefix] + M_out[prefix];
              ++prefix;
            }
            cv.notify_all();
            cv.wait(lk, [&] { return prefix > t; });
          }
          if (rc != DS_OK) continue;
          if (offsets[t + 1] > capacity) {  // no room for this one: its size is reported, nothing is written
            ds_cgraph_free(w, cg);
            continue;
          }
          int64_t m = M_out[t];
          const int64_t off = offsets[t];
          status[t] = explain_extracted(w, cg, targets[t], n_samples, seed, o, phi_concat ? phi_concat + off : nullptr, &m,
                                        edge_src ? edge_src + off : nullptr, edge_dst ? edge_dst + off : nullptr,
                                        reports ? reports + t : nullptr);
          if (status[t] != DS_OK && status[t] != DS_ENOTCONV) errs[t] = w->err;
        }
      });
    for (auto& th : pool) th.join();
  }
  int worst = offsets[num_targets] > capacity ? DS_ECAPACITY : DS_OK;
  if (worst == DS_ECAPACITY)
    ds_fail(ctx, DS_ECAPACITY, "the batch needs %lld entries, the buffers hold %lld", (long long)offsets[num_targets], (long long)capacity);
  for (int32_t t = 0; t < num_targets; ++t) {
    if (status[t] == DS_ENOTCONV) {
      if (worst == DS_OK) worst = DS_ENOTCONV;
    } else if (status[t] != DS_OK) {
      strncpy(ctx->err, errs[t].c_str(), sizeof(ctx->err) - 1);
      return status[t];
    }
  }
  return worst;
}

}  // extern "C"
