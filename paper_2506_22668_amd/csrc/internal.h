// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include <string.h>
#include <vector>

#include "../../include/distshap.h"

#define DS_MAX_LAYERS 7
#define DS_MAX_HOPS 7
#define DS_ENUM_MAX_PLAYERS 24
#define DS_WAVE 64
#define DS_MAX_DEVICES 64
#define DS_EVAL_NOALLOC_SCRATCH_BYTES (32u << 20)

struct ds_cgraph {
  ds_ctx* owner;
  ds_cgraph_info info;
  void* block;            // one device allocation holding every array below
  size_t block_bytes;
  int32_t* row_ptr;       // [V+1] local CSR, row t lists local in-neighbours
  int32_t* col;           // [nnz]
  int32_t* eid;           // [nnz] CSR entry -> player
  int2* pl;               // [n] player end points as local ids: x = a (undirected: the smaller global id) or the
                          // message source, y = b or the message destination
  int64_t* node_gid;      // [V]
  int32_t* hop;           // [V]
  float* Xc;              // [V x d0] gathered feature rows
  float* P;               // [V x d1] shared first transform Xc * W_1 (valid if model_version matches)
  float* att;             // GAT only: layer-1 attention scalars, neighbour part [V x heads_1] then receiver part
  int32_t* d_pred;        // device: class predicted on the full graph (valid with model_version)
  uint64_t model_version; // model the cached P / d_pred belong to (0 = none)
  int32_t pred_class;     // host copy, -1 until fetched
  int32_t d0, d1;
  int64_t ball_entries[8]; // row_ptr[ball[h]]: CSR entries of the rows within h hops
  int32_t att_heads;       // heads the `att` array was sized for (0: extracted for a GCN)
};

#define DS_MODEL_GCN 0
#define DS_MODEL_GAT 1

// attention parameters of a GAT (model_kind == DS_MODEL_GAT); dims[] of the context then holds the width
// of every layer's OUTPUT (heads * head width for a hidden layer, head width for the last one)
struct ds_gat_params {
  int32_t heads[DS_MAX_LAYERS];
  int32_t fh[DS_MAX_LAYERS];  // per-head width
  int32_t zw[DS_MAX_LAYERS];  // heads * fh: width of the layer's dense transform
  const float* att_src[DS_MAX_LAYERS];
  const float* att_dst[DS_MAX_LAYERS];
  float slope;
};

// The small members of sparse complementary pairs as player lists, written by the sampler beside the mask rows
// (a row with s of n players set is 4 s bytes as a list and n / 8 bytes as a bit row): pair r's players, in no
// particular order, are entries[offset[r] .. offset[r] + s), offset[r] < 0 where the pair has no list (a size class
// above max_size, an enumerated class, a pair the one-pass sampler handed on).
struct ds_pair_lists {
  uint32_t* entries;   // device
  int64_t* offset;     // device, [pairs]
  int64_t max_size;    // size classes 1..max_size are listed
  int64_t total;       // entries reserved
};

struct ds_ctx {
  int device;
  hipStream_t stream;
  char err[512];
  // graph and features (caller-owned device memory)
  int64_t N, nnz;
  const int64_t* row_ptr;
  const int32_t* col;
  const float* X;
  int32_t d0;
  // model
  int32_t L;
  int32_t dims[DS_MAX_LAYERS + 1];
  const float* W[DS_MAX_LAYERS];
  const float* bias[DS_MAX_LAYERS];
  int32_t transform_dtype;
  uint64_t model_version;
  int32_t model_kind;
  ds_gat_params gat;
  // bump arena for temporaries (grown only while nothing is live)
  char* arena;
  size_t arena_bytes, arena_used;
  // small device<->host mailbox
  int64_t* d_mail;  // device int64[64]
  int64_t* h_mail;  // pinned host int64[64]
  int num_cus;
  hipEvent_t ev[6];
  hipEvent_t kev[10];  // begin/end pairs: 0 masked inference, 1 Gram, 2 Cholesky, 3 CGLS loop, 4 mask-streaming kernel
  bool kev_set[5];
  std::vector<ds_cgraph*> graphs;
  // one released computational-graph block is kept for the next extraction (no malloc/free per explanation)
  void* cg_spare;
  size_t cg_spare_bytes;
  // pinned staging for the sampling plan tables, and the event that says the last upload from it is done
  char* h_stage;
  size_t h_stage_bytes;
  hipEvent_t stage_ev;
  bool stage_busy;
  // a second stream (default priority) for work that does not depend on what the main stream is doing
  hipStream_t side;
  hipEvent_t fork_ev, join_ev, fork2_ev, join2_ev;
  // ds_explain_batch runs several targets at once on worker contexts (own stream, own workspace)
  std::vector<ds_ctx*> workers;
  bool owns_stream;
  ds_tuning tuning;  // zero fields = built-in values
  double cgls_bytes_per_iter;  // bytes of matrix storage the last CGLS solve read per iteration (both products)
  ds_pair_lists lists;         // set by an explanation between its sampling and its inference; entries == nullptr: none
};

int ds_fail(ds_ctx* ctx, int code, const char* fmt, ...);

#define DS_HIP(ctx, call)                                                                   \
  do {                                                                                      \
    hipError_t e__ = (call);                                                                \
    if (e__ != hipSuccess)                                                                  \
      return ds_fail(ctx, DS_EDEVICE, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e__), \
                     __FILE__, __LINE__);                                                   \
  } while (0)

#define DS_TRY(expr)            \
  do {                          \
    int rc__ = (expr);          \
    if (rc__ != DS_OK) return rc__; \
  } while (0)

// arena
int ds_arena_reserve(ds_ctx* ctx, size_t bytes);  // only when arena_used == 0
void* ds_arena_alloc(ds_ctx* ctx, size_t bytes);  // nullptr when exhausted
static inline void ds_arena_reset(ds_ctx* ctx) { ctx->arena_used = 0; }
static inline size_t ds_align(size_t b) { return (b + 255) & ~(size_t)255; }
// record the begin (end=0) or end (end=1) event of kernel slot `slot`
int ds_kernel_mark(ds_ctx* ctx, int slot, int end);
// copy `count` int64 values from the device mailbox to the host mailbox (synchronises)
int ds_mail_fetch(ds_ctx* ctx, int count);

// ---- stages (host drivers; each launches its kernels on ctx->stream) ----
struct ds_plan {
  int64_t n, k, K, H;
  int enumerate;
  int64_t enum_upto;        // size classes 1..enum_upto are enumerated (every subset once), the rest sampled
  std::vector<int64_t> b;   // class boundaries b[0..H]
  std::vector<float> wtab;  // weight per pair class, wtab[0..H]
};
int ds_make_plan(ds_ctx* ctx, int64_t n, int64_t n_samples, ds_plan* plan, int weighting = DS_WEIGHT_CLASS_MASS,
                 int saturate = 0);
// launches the sampler; the overflow flag is left in device mailbox slot DS_MAIL_SAMPLER (checked by the caller)
// lists (optional, only with pair_begin == 0): filled as described at ds_pair_lists; entries and offset are the
// caller's allocations (ds_pair_list_entries(plan, max_size) entries, plan.k / 2 offsets)
int ds_sample_launch(ds_ctx* ctx, const ds_plan& plan, uint64_t seed, uint32_t tag, int64_t pair_begin,
                     int64_t pair_end, uint64_t* Z, float* w, int32_t* sz, const ds_pair_lists* lists = nullptr);
int64_t ds_pair_list_entries(const ds_plan& plan, int64_t max_size);
// whether the sampler can write lists for this plan at all (the one-pass kernel runs)
bool ds_sampler_lists_possible(const ds_ctx* ctx, const ds_plan& plan);
// whether ds_eval_impl would run the mask-streaming kernel on k paired rows of this graph (the consumer of the lists)
bool ds_eval_streams_pairs(ds_ctx* ctx, const ds_cgraph* cg, int64_t k);
int ds_sample_check(ds_ctx* ctx);  // synchronises and turns the flag into a status
#define DS_MAIL_SAMPLER 20
int ds_fetch_pred_class(ds_ctx* ctx, ds_cgraph* cg);  // device -> host copy of the predicted class (synchronises)
size_t ds_sample_arena_bytes(const ds_plan& plan);

int ds_scan_exclusive_i32(ds_ctx* ctx, const int32_t* in, int32_t* out, int64_t count, int64_t* total_mail_slot);
size_t ds_scan_arena_bytes(int64_t count);

int ds_extract_impl(ds_ctx* ctx, int64_t target, int hops, int directed, ds_cgraph** out);
int ds_validate_csr(ds_ctx* ctx);

#define DS_EVAL_BOUNDED 1  // the workspace is not the context's own arena: fit the launch into what is there
#define DS_EVAL_PAIRED 2   // rows 2r, 2r+1 are complementary pairs: only row 2r of each is read
// sz: coalition size of every row (the sampler's output) or nullptr
int ds_eval_impl(ds_ctx* ctx, ds_cgraph* cg, const uint64_t* Z, int64_t k, int score, float* y, int flags,
                 const int32_t* sz = nullptr);
int ds_prepare_model(ds_ctx* ctx, ds_cgraph* cg);  // shared first transform + predicted class
// the file-scope device array behind ds_eval_noalloc: address look-up (once per device, that device current)
// and the pointer found
int ds_static_scratch_init(int device);
void* ds_static_scratch(int device);
size_t ds_eval_arena_bytes(ds_ctx* ctx, const ds_cgraph* cg, int64_t k);
// masked GCN inference layer by layer over blocks of 64 coalitions from a block-transposed mask matrix (graphs whose
// first layer reads too many entries for the on-chip kernels); the model must be prepared
bool ds_eval_zt_applies(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k, int64_t min_rows = 256);
size_t ds_eval_zt_arena_bytes(const ds_ctx* ctx, const ds_cgraph* cg, int64_t k, int64_t min_rows = 256);
// logits_out: optional [k x d_L]; pred_ptr: device, the class whose score goes to y; paired: rows 2r, 2r+1 are complements
int ds_eval_zt(ds_ctx* ctx, ds_cgraph* cg, const uint64_t* Z, int64_t k, int score, float* y, float* logits_out,
               const int32_t* pred_ptr, int paired = 0);
// width of the shared first transform P = X_c W_1
static inline int32_t ds_first_width(const ds_ctx* ctx) {
  if (ctx->L < 1) return 0;
  return ctx->model_kind == DS_MODEL_GAT ? ctx->gat.zw[0] : ctx->dims[1];
}
// small launchers shared by the two model families (defined next to the GCN kernels)
int ds_launch_first_transform(ds_ctx* ctx, const float* A, const float* B, float* C, int M, int K, int Nn, int bf16);
int ds_launch_full_mask(ds_ctx* ctx, uint64_t* z, int64_t W, int64_t n);
int ds_launch_argmax(ds_ctx* ctx, const float* logits, int C, int32_t* out);
// GAT counterparts of the three functions above (same contracts)
int ds_gat_prepare_model(ds_ctx* ctx, ds_cgraph* cg);
int ds_gat_eval_impl(ds_ctx* ctx, ds_cgraph* cg, const uint64_t* Z, int64_t k, int score, float* y);
size_t ds_gat_eval_arena_bytes(ds_ctx* ctx, const ds_cgraph* cg, int64_t k);

// the direct solver in two parts: the first needs only the masks and weights
struct ds_gram_state {
  int64_t n, k, R, RW, ld, nblk;
  int paired;
  uint64_t* Zt;
  double *M, *linv, *t, *sqw, *gc, *c, *yv;
  double* panel[2];  // rows of the current and of the next 64-column panel (fused steps of the factorisation)
  int32_t* sz;
  float* wc;
  int* flag;
};
int ds_gram_begin(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, int paired, ds_gram_state* gs);
// defer_check != 0: the non-positive-pivot flag (gs->flag, device int) is left for the caller to read back
int ds_gram_finish(ds_ctx* ctx, const ds_gram_state* gs, const uint64_t* Z, const float* w, const float* y, float* phi,
                    int defer_check);
int ds_solve_gram_chol(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, const float* y,
                       int paired, float* phi);
size_t ds_gram_arena_bytes(int64_t n, int64_t k);
int ds_solve_cgls_impl(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, const float* y,
                       int paired, double tol, int max_iter, float* phi, int* iters, double* relres);
size_t ds_cgls_arena_bytes(int64_t n, int64_t k);
