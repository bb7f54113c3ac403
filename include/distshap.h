/*
 * distshap.h - C ABI of the MI355X (gfx950) Kernel-SHAP edge-attribution library.
 *
 * The library computes, on one GPU, the hot path of DistShap (arxiv 2506.22668):
 * for a target node v of a graph and a trained GCN f, the players of the game are
 * the edges of v's computational graph G_c(v) (paper, "Overview of DistShap",
 * step 1), coalitions are sampled as rows of a binary mask matrix ("Distributed
 * Subgraph Sampling"), f is evaluated on every masked sub-graph ("Distributed
 * Model Prediction"), and the Shapley-kernel weighted least-squares problem is
 * solved for one score per edge ("Distributed Shapley Computations", Alg. 1).
 *
 * Conventions
 *  - Plain C; every call returns an int status (DS_OK == 0). No exception crosses
 *    the boundary. ds_last_error() gives a human-readable message for the last
 *    failing call on that context.
 *  - Unless a parameter is marked [host], pointers are DEVICE pointers on the
 *    context's GPU. The caller owns every buffer it passes in; the library never
 *    frees them and keeps pointers only for the ds_set_* calls (those buffers
 *    must stay valid and unchanged until the context is destroyed or re-set).
 *  - All work is issued on the context's stream; calls that return host values
 *    synchronise that stream before returning.
 *  - A context is not thread-safe; use one per thread.
 *  - Player order (bit j of a mask row <-> player j <-> phi[j]):
 *      undirected: unordered node pairs {a < b} (global ids) joined by an edge
 *                  with both ends in G_c(v), ascending by (a, b);
 *      directed:   CSR entries (dst, src), src != dst, both ends in G_c(v),
 *                  ascending by (dst, src).
 *  - Mask rows are bit-packed: row i occupies W = ceil(n/64) uint64 words at
 *    Z[i*W .. i*W+W-1]; player j is bit (j & 63) of word (j >> 6); padding bits
 *    are zero.
 */
#ifndef DISTSHAP_H
#define DISTSHAP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ds_ctx ds_ctx;       /* library context (device, stream, model, workspace) */
typedef struct ds_cgraph ds_cgraph; /* an extracted computational graph, owned by the library */

enum ds_status {
  DS_OK = 0,
  DS_EINVAL = 1,    /* bad argument, malformed or asymmetric CSR, n_samples too small */
  DS_ECAPACITY = 2, /* an output buffer is too small; the needed size is written back */
  DS_ENOMEM = 3,    /* device allocation failed */
  DS_ENOTCONV = 4,  /* CGLS stopped at max_iter; phi holds the last iterate */
  DS_EDEVICE = 5,   /* a HIP call failed */
  DS_ESINGULAR = 6, /* Cholesky met a non-positive pivot (Gram matrix rank-deficient) */
  DS_EINTERNAL = 7  /* an internal capacity was exceeded; no result was produced */
};

enum ds_dtype {
  DS_F32 = 0,            /* fp32 storage and arithmetic */
  DS_BF16_IN_F32_ACC = 1 /* the per-coalition dense transforms (layers 2..L) round both operands to bf16 and
                            accumulate in fp32; the product X_c W_1, formed once per target, stays fp32 */
};

enum ds_score { DS_SCORE_PROB = 0, DS_SCORE_LOGIT = 1 };
enum ds_solver { DS_SOLVER_AUTO = 0, DS_SOLVER_GRAM_CHOL = 1, DS_SOLVER_CGLS = 2 };
/* Regression weight of a sampled row (paper, "Shapley value" / sample-distribution equation: rho_s is the
 * total kernel weight of the coalitions of size s and the rows are allocated in proportion to it).
 * CLASS_MASS: a row of size s weighs rho_s / (rows of size s), so every represented size carries its whole
 * mass. UNIFORM: every sampled row weighs 1, the importance-sampling form of the same estimator (the two
 * differ through the rounding of the allocation and the classes that received no row). Enumerated
 * explanations always use the exact kernel weights. */
enum ds_weighting { DS_WEIGHT_CLASS_MASS = 0, DS_WEIGHT_UNIFORM = 1 };

/* Options of an explanation. Zero-initialise for the defaults. */
typedef struct ds_options {
  int32_t hops;       /* radius of the computational graph; 0 -> number of GCN layers */
  int32_t directed;   /* 0: a player is an undirected edge (both CSR entries); 1: one CSR entry */
  int32_t score;      /* ds_score: softmax probability (default) or raw logit of the class
                         predicted on the full computational graph */
  int32_t solver;     /* ds_solver; AUTO picks GRAM_CHOL for n <= 16384, else CGLS */
  double tol;         /* CGLS: stop when |s_i| / |s_0| <= tol; 0 -> 1e-6 */
  int32_t max_iter;   /* CGLS: 0 -> min(n, 10000) */
  int32_t batch_rows; /* reserved (one launch covers all coalition rows); leave 0 */
  int32_t paired;     /* ds_solve only: 1 promises that rows 2r and 2r+1 are complements with
                         equal weights (the layout ds_sample writes), which lets CGLS read only
                         one member of each pair; 0 makes no assumption. ds_explain always
                         uses its own paired rows. */
  int32_t weighting;  /* ds_weighting, honoured by ds_explain, ds_explain_batch, ds_sample_ex and
                         ds_plan_tables_ex (ds_sample / ds_plan_tables always use CLASS_MASS) */
  int32_t saturate;   /* 1: a size class that is allotted at least as many pairs as it has coalitions
                         (q_s >= C(n, s); the sizes 1 and n-1 on small graphs) is enumerated instead of
                         sampled: its pairs are the s-subsets of the players in lexicographic order, each once,
                         weighted by the Shapley kernel itself, and the pairs this frees go to the other
                         classes by the same allotment rule. Needs CLASS_MASS weighting. Honoured where
                         `weighting` is. 0 (default): every class is sampled. */
} ds_options;

/* What an explanation did (all [host]). Times are wall-clock milliseconds measured
 * with HIP events on the context's stream. */
typedef struct ds_report {
  int64_t num_players;    /* n */
  int64_t num_nodes;      /* |V_c| */
  int64_t num_entries;    /* directed CSR entries of G_c (self-loops excluded) */
  int64_t num_rows;       /* k: rows of the mask matrix actually used */
  int32_t enumerated;     /* 1 if all 2^n coalitions were enumerated */
  int32_t pred_class;     /* class predicted on the full computational graph */
  int32_t solver_used;    /* ds_solver */
  int32_t cgls_iterations;
  double cgls_rel_residual; /* |s_i| / |s_0| at exit */
  double f_empty;         /* f(no edges) = phi_0 */
  double f_full;          /* f(all edges) */
  float ms_extract, ms_sample, ms_eval, ms_solve, ms_total;
  /* single-kernel durations inside the stages above (0 when the kernel did not run):
   * the masked-inference kernel over all k rows, the popcount Gram kernel, the
   * Cholesky factorisation launches, and the CGLS loop (all iterations). */
  float ms_k_eval, ms_k_gram, ms_k_chol, ms_k_cgls;
  int64_t num_pairs;      /* K: sampled complementary pairs (rows 2..k-1 are K pairs; 2^(n-1) - 1 when enumerated) */
  /* Algorithmic bytes of each stage: what the step has to move whatever the kernel does, the basis of the
   * roofline fractions (W = ceil(n/64) words per mask row).
   *   sample: k*W*8 mask bytes + k*8 bytes of weights and sizes written;
   *   eval:   one member of every complementary pair read (the other is its complement and needs no second
   *           look), (k/2)*W*8, plus k*4 bytes of outputs;
   *   solve:  CGLS: per iteration the small member of every pair once for Z u and once for Z^T r, in the storage
   *           the solver keeps them in: iterations * 2 * (bit-packed rows * W*8 + 4 bytes per set bit of the rows
   *           kept as (row, column) entries); all rows bit-packed for games below 4,096 players. Gram + Cholesky:
   *           (k/2)*W*8 mask bytes read, n*n*4 bytes of Gram matrix written. */
  double bytes_sample, bytes_eval, bytes_solve;
  float ms_k_stream;      /* the mask-streaming kernel alone (long mask rows; part of ms_k_eval), else 0 */
} ds_report;

typedef struct ds_cgraph_info {
  int64_t num_players;
  int64_t num_nodes;
  int64_t num_entries;
  int64_t target;    /* global id */
  int32_t hops;
  int32_t directed;
  int64_t ball[8];   /* ball[h] = number of nodes within h hops, h = 0..hops (hops <= 7) */
} ds_cgraph_info;

/* ---- context --------------------------------------------------------------- */

/* Create a context on HIP device `device`. `stream` is a hipStream_t passed as
 * void* (NULL = the default stream). [host] out. */
int ds_create(ds_ctx** out, int device, void* stream);
/* Release the context, its workspace and every computational graph still alive. */
int ds_destroy(ds_ctx* ctx);
/* Message of the last failing call on this context (static storage, [host]). */
const char* ds_last_error(const ds_ctx* ctx);

/* Tuning of a context (none of it changes a result). Zero in a field keeps the built-in value, which is the
 * measured optimum; pass NULL to restore all of them. Worker contexts of ds_explain_batch inherit the values. */
typedef struct ds_tuning {
  int32_t batch_workers;      /* explanations in flight in ds_explain_batch, 1..16 (default 8) */
  int32_t gram_sparse_div;    /* Gram: rows with at most n / div set columns are accumulated row-wise (default 12) */
  float gram_dense_fraction;  /* Gram: density from which a 64-row word with mixed weights goes to the matrix
                                 cores (default 0.08) */
  int32_t sampler_window;     /* sampler: capacity (entries) of the list of keys the first pass keeps around the
                                 expected threshold; -1 keeps none. A small list forces the slower four-pass
                                 selection (a test hook: the masks are the same either way) */
  int32_t eval_path;          /* masked GCN inference kernel: 0 = chosen by size; 1 = one workgroup per coalition;
                                 2 = one coalition per lane, masks on chip (short mask rows); 3 = the mask-streaming
                                 kernel followed by the one-coalition-per-lane layers (long mask rows); 4 = layer by
                                 layer over blocks of 64 coalitions from a transposed mask matrix (graphs whose first
                                 layer reads more entries than fit on chip). 2, 3 and 4 need 256 rows or more and fall
                                 back to 1 where they do not apply (a test hook: the results agree to rounding) */
  int32_t cgls_dense_div;     /* CGLS on large games: pair rows with more than n / div players stay bit-packed and
                                 are multiplied on the int8 matrix cores, the sparser ones become (row, column)
                                 entries multiplied through LDS (default 64, the measured optimum; 32..65536) */
  int32_t pair_lists;         /* ds_explain with long mask rows: the sampler also writes the players of every sparse
                                 small member (at most n / div players; 0 = default div 64, a list of half the bit row's
                                 bytes; 16..2^20) as a list, which the mask-streaming kernel reads instead of
                                 the bit row; -1 = bit rows only (a test hook: the results are identical) */
} ds_tuning;
int ds_set_tuning(ds_ctx* ctx, const ds_tuning* tuning /* [host] or NULL */);

/* Graph G(V, E) as a CSR adjacency (paper, "Background & Related Work"): row i
 * lists the in-neighbours j of node i (messages flow j -> i), strictly ascending,
 * ids in [0, N). row_ptr: int64[N+1], col: int32[row_ptr[N]]. Self-loop entries
 * are allowed and ignored. The structure is validated on the device; a malformed
 * CSR gives DS_EINVAL. */
int ds_set_graph(ds_ctx* ctx, int64_t num_nodes, const int64_t* row_ptr, const int32_t* col);

/* Node features X, row-major [N x d0], fp32 (dtype must be DS_F32). */
int ds_set_features(ds_ctx* ctx, const void* X, int32_t d0, int32_t dtype);

/* GCN weights (paper, "GNN Models": L-layer GCN with ReLU; layer rule of Kipf &
 * Welling with degrees renormalised for every coalition):
 *   H^l = ReLU(A^_S H^(l-1) W_l + b_l), no ReLU on layer L.
 * dims [host]: int32[L+1] = d0..dL. W [host]: array of L device pointers, W_l
 * row-major fp32 [d_(l-1) x d_l]. bias [host]: NULL, or array of L device
 * pointers (entries may be NULL) to fp32[d_l]. 1 <= L <= 7, dL <= 1024.
 * transform_dtype: ds_dtype applied to the dense transforms. */
int ds_set_gcn(ds_ctx* ctx, int32_t num_layers, const int32_t* dims, const void* const* W,
               const void* const* bias, int32_t transform_dtype);

/* GAT weights (paper, "GNN Models" and the GAT scaling experiment: a two-layer
 * graph attention network with 8 heads; layer rule of Velickovic et al., which
 * the paper cites). Replaces the model set by ds_set_gcn (and vice versa).
 * Layer l has heads[l-1] heads of width head_dims[l]; with Z = H^(l-1) W_l and
 * z_i^h the h-th slice of row i, on the sub-graph of coalition S
 *   e_ij^h = LeakyReLU(att_dst_l^h . z_i^h + att_src_l^h . z_j^h),  j in N_S(i) + {i},
 *   alpha_ij^h = softmax_j(e_ij^h),   out_i^h = sum_j alpha_ij^h z_j^h;
 * a hidden layer concatenates its heads, adds b_l and applies ELU, the last
 * layer averages its heads and adds b_L. The self term is always present.
 * head_dims [host]: int32[L+1] = d0, then the per-head width of every layer
 * (the last is the number of classes). heads [host]: int32[L].
 * W [host]: L device pointers, W_l row-major fp32 [in_l x heads_l*head_dims_l]
 * with in_1 = d0 and in_l = heads_(l-1)*head_dims_(l-1). att_src, att_dst
 * [host]: L device pointers each, fp32 [heads_l x head_dims_l] (att_dst
 * multiplies the receiving node, att_src the neighbour). bias [host]: NULL, or
 * L device pointers (entries may be NULL) to fp32[heads_l*head_dims_l] (hidden)
 * or fp32[head_dims_L] (last). 1 <= L <= 7; transform widths <= 4096, classes
 * <= 1024. fp32 arithmetic throughout. */
int ds_set_gat(ds_ctx* ctx, int32_t num_layers, const int32_t* head_dims, const int32_t* heads,
               const void* const* W, const void* const* att_src, const void* const* att_dst,
               const void* const* bias, float negative_slope);

/* ---- one-shot explanation --------------------------------------------------- */

/* Explain the prediction for `target`: extract G_c, draw n_samples coalitions
 * (seeded; identical (seed, target, n) always give the same masks), evaluate the
 * GCN on each, solve for phi.
 *   phi:       float[capacity]  out, phi[j] = attribution of player j
 *   M_inout:   [host] in: capacity of phi / edge_src / edge_dst; out: n
 *   edge_src, edge_dst: int64[capacity] out or NULL, global ids of the players
 *   report:    [host] out or NULL
 * n == 0 is a success with *M_inout = 0. n_samples < 4 is DS_EINVAL when n >= 2.
 * DS_ECAPACITY writes the needed n to *M_inout and touches no output buffer. */
int ds_explain(ds_ctx* ctx, int64_t target, int64_t n_samples, uint64_t seed, const ds_options* opts,
               float* phi, int64_t* M_inout, int64_t* edge_src, int64_t* edge_dst, ds_report* report);

/* Explain T targets (paper's protocol: a set of test nodes per run). Every target gets exactly the result
 * ds_explain would give it; up to eight explanations are in flight at a time (two when the games average more
 * than 4096 players, one above 16384), each on an internal worker context with its own stream, workspace and
 * host thread, which fills the GPU better than one small explanation at a time. The call returns when all are done.
 *   targets [host]: int64[T]; phi_concat: float[capacity] out, target t's scores at
 *   offsets[t] .. offsets[t+1]-1; M_out [host]: int64[T]; offsets [host]: int64[T+1];
 *   edge_src/edge_dst: int64[capacity] or NULL; reports [host]: ds_report[T] or NULL.
 * If the total exceeds `capacity`, DS_ECAPACITY is returned, M_out and offsets are complete
 * (offsets[T] is the needed total) and the targets whose range fits are explained. */
int ds_explain_batch(ds_ctx* ctx, const int64_t* targets, int32_t num_targets, int64_t n_samples,
                     uint64_t seed, const ds_options* opts, float* phi_concat, int64_t* M_out,
                     int64_t* offsets, int64_t* edge_src, int64_t* edge_dst, int64_t capacity,
                     ds_report* reports);

/* ---- stage-wise calls (the same kernels, exposed for parity checks) ---------- */

/* Computational graph of `target` (paper: the L-hop neighbourhood and the edges
 * among its nodes). Local node order: ascending (hop, global id). *out [host] is
 * owned by the library; release with ds_cgraph_free. Uses opts->hops/directed. */
int ds_extract(ds_ctx* ctx, int64_t target, const ds_options* opts, ds_cgraph** out);
int ds_cgraph_get_info(const ds_cgraph* cg, ds_cgraph_info* info /* [host] */);
/* Copy out the player list (global ids; undirected: src = a < dst = b). int64[n] each, may be NULL. */
int ds_cgraph_edges(ds_ctx* ctx, const ds_cgraph* cg, int64_t* edge_src, int64_t* edge_dst);
/* Copy out node_gid int64[|V_c|] and hop int32[|V_c|] in local order (either may be NULL). */
int ds_cgraph_nodes(ds_ctx* ctx, const ds_cgraph* cg, int64_t* node_gid, int32_t* hop);
/* Copy out the shared first-layer product X_c W_1 (paper's |V_c| d^2 term, computed once per
 * target on the matrix cores): float[|V_c| x d_1], local node order. */
int ds_cgraph_first_transform(ds_ctx* ctx, ds_cgraph* cg, float* out);
int ds_cgraph_free(ds_ctx* ctx, ds_cgraph* cg);

/* Number of mask rows k that n_samples yields for n players, and whether all
 * coalitions are enumerated (n <= 24 and n_samples >= 2^n). Pure host function.
 * k = 2*floor(n_samples/2) otherwise. [host] outputs. */
int ds_sample_plan(int64_t n, int64_t n_samples, int64_t* k_out, int32_t* enumerated_out);

/* The size-stratified allocation behind ds_sample (paper, sample-distribution equation: the samples of
 * size s are proportional to rho_s = (n-1)/(s(n-s)); complementary pairing). Pure host function, all
 * [host]: for pair classes s = 1..H, H = floor(n/2), writes the cumulative pair boundaries b[0..H]
 * (pair r in [1, K] has small size min{s : b[s] >= r}; all zero under enumeration) and the per-row
 * regression weight wtab[0..H] of a row of size s or n-s. Either output may be NULL. n >= 2. */
int ds_plan_tables(int64_t n, int64_t n_samples, int64_t* b, float* wtab);

/* ds_plan_tables with the options that change the plan (weighting, saturate). enum_upto [host] (may be NULL):
 * the size classes 1..enum_upto are enumerated. */
int ds_plan_tables_ex(int64_t n, int64_t n_samples, const ds_options* opts, int64_t* b, float* wtab,
                      int64_t* enum_upto);

/* Sampler (paper, "Distributed Subgraph Sampling": size-stratified allocation by
 * the kernel mass of each size, complementary pairs, one mask row per coalition).
 * Row 0 is the empty and row 1 the full coalition (weight 0: they are imposed as
 * constraints); pair r >= 1 is rows 2r (small member) and 2r+1 (complement), pairs
 * ascending by size. Random keys come from Philox4x32-10 with key = seed and
 * counter (column/4, r, tag), so any pair range can be regenerated alone.
 *   Z: uint64[k*W] out; w: float[k] out (per-row regression weight);
 *   sz: int32[k] out (coalition sizes); k_out [host]. tag: stream id (the
 *   explanation uses the low 32 bits of the target's global id).
 */
int ds_sample(ds_ctx* ctx, int64_t n, int64_t n_samples, uint64_t seed, uint32_t tag, uint64_t* Z,
              float* w, int32_t* sz, int64_t* k_out);
/* ds_sample with the options that change the plan (opts->weighting, opts->saturate; NULL = defaults). */
int ds_sample_ex(ds_ctx* ctx, int64_t n, int64_t n_samples, uint64_t seed, uint32_t tag, const ds_options* opts,
                 uint64_t* Z, float* w, int32_t* sz, int64_t* k_out);
/* Only pairs pair_begin <= r < pair_end: writes rows 2*pair_begin .. 2*pair_end-1
 * to Z[0..], w[0..], sz[0..] (what one GPU of a sharded run would generate). */
int ds_sample_range(ds_ctx* ctx, int64_t n, int64_t n_samples, uint64_t seed, uint32_t tag,
                    int64_t pair_begin, int64_t pair_end, uint64_t* Z, float* w, int32_t* sz);

/* Masked GCN inference (paper, "Distributed Model Prediction"): y[i] = f(S_i) for
 * the k coalitions in Z (any rows, not necessarily paired), using the context's
 * features and GCN. y: float[k] out. score: ds_score. pred_class_out [host] may be
 * NULL. */
int ds_eval(ds_ctx* ctx, const ds_cgraph* cg, const uint64_t* Z, int64_t k, int32_t score, float* y,
            int32_t* pred_class_out);

/* ds_eval for rows that come in complementary pairs, the layout ds_sample writes (paper, "Distributed Subgraph
 * Sampling": paired sampling): row 2r+1 must be the complement of row 2r on the n players; k even. Only row 2r of
 * each pair is read (the complement's degrees and entry bits follow from it), which halves the mask traffic of
 * long rows. Results equal ds_eval's. Rows that are not complements give undefined y for the odd rows. */
int ds_eval_pairs(ds_ctx* ctx, const ds_cgraph* cg, const uint64_t* Z, int64_t k, int32_t score, float* y,
                  int32_t* pred_class_out);

/* ds_eval for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc. Same kernels and results as ds_eval, but every byte of scratch memory comes
 * from an array of 32 MiB that is part of the library's device image (each GPU the library runs on holds its own
 * copy until the process ends; its address is looked up once per device in ds_create). The call allocates and
 * frees nothing and does not synchronise: work is queued on the context's stream and y is valid once that
 * stream has reached it. GCN only. When the scratch of one workgroup does not fit the array the launch uses
 * fewer workgroups; when not even one fits (or the mask row itself is too wide: beyond about 2.6e8 players)
 * DS_ECAPACITY is returned and nothing runs. All calls on one GPU share the one array, from any context or
 * thread: calls that overlap in time on a GPU race on it, so the caller serialises them (one stream, or events).
 * Nothing in the array has to start at zero. The class whose score is returned is the one predicted on the
 * full graph, as in ds_eval; it is not copied to the host here (ds_eval does that). */
int ds_eval_noalloc(ds_ctx* ctx, const ds_cgraph* cg, const uint64_t* Z, int64_t k, int32_t score, float* y);

/* Constrained weighted least squares (paper, Eq. for Kernel-SHAP regression, the
 * efficiency decomposition, and Alg. 1): rows 0/1 of Z must be the empty/full
 * coalitions; phi minimises sum_{i>=2} w_i (y_i - y_0 - z_i.phi)^2 subject to
 * sum(phi) = y_1 - y_0; when rank-deficient the solution closest to the uniform
 * split is returned (CGLS only). phi: float[n] out. report [host] may be NULL
 * (fills solver_used, cgls_*). */
int ds_solve(ds_ctx* ctx, int64_t n, int64_t k, const uint64_t* Z, const float* w, const float* y,
             const ds_options* opts, float* phi, ds_report* report);

/* Top-k explanation sub-graph and its fidelity (paper, overview step 5 and the evaluation-metric
 * equations): for each k = topk[t], G_s = the k players with the largest phi (ties to the lower
 * index), fid_plus[t] = |f(G_c) - f(G_c \ G_s)|, fid_minus[t] = |f(G_c) - f(G_s)|, with f the masked
 * GCN inference of ds_eval. phi: float[n] (device). topk [host]: int64[num_k], values outside [0, n]
 * are clamped. fid_plus, fid_minus [host]: float[num_k] out. masks_out: NULL, or uint64[2*num_k*W]
 * (device) receiving row 2t = G_s and row 2t+1 = its complement. 1 <= num_k <= 4096. */
int ds_fidelity(ds_ctx* ctx, const ds_cgraph* cg, const float* phi, const int64_t* topk, int32_t num_k,
                int32_t score, float* fid_plus, float* fid_minus, uint64_t* masks_out);

/* Measurement aid: a plain device-to-device copy of `bytes` bytes (multiple of 16) by a simple
 * streaming kernel on the context's stream. Profilers' HBM byte counters are calibrated against it
 * (its traffic is exactly `bytes` read and `bytes` written). dst and src must not overlap. */
int ds_copy_probe(ds_ctx* ctx, void* dst, const void* src, int64_t bytes);

/* Library version string ([host], static). */
const char* ds_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DISTSHAP_H */
