// Helpers shared by the two least-squares solvers (internal).
#pragma once
#include "internal.h"

// sz[i] = |S_i|, t[i] = y_i - y_0 - ((y_1-y_0)/n)|S_i| (0 for the two constraint rows),
// sqw[i] = sqrt(w_i), wc[i] = w_i (both 0 for the two constraint rows)
int ds_row_prep(ds_ctx* ctx, const uint64_t* Z, int64_t k, int64_t n, const float* w, const float* y, int32_t* sz,
                double* t, double* sqw, float* wc);
// out[cols x ceil(rows/64)] = transpose of the rows row_first + i*row_step (i < rows) of `in`
int ds_bit_transpose(ds_ctx* ctx, const uint64_t* in, int64_t rows, int64_t cols, int64_t in_stride, int64_t row_first,
                     int64_t row_step, uint64_t* out);
// the same transpose of the rows i * row_step (i < rows), laid out by blocks of 64 of them: out[b * 64*ceil(cols/64) + j] =
// bits of column j in the rows 64b .. 64b+63 of that selection (rows past the last and columns past `cols` read as zero)
int ds_bit_transpose_blocks(ds_ctx* ctx, const uint64_t* in, int64_t rows, int64_t cols, int64_t in_stride, int64_t row_step,
                            uint64_t* out);
// out[i] = sum of x[j] over the set bits j < cols of row (row_first + i*row_step) of B, i < rows (fp64)
int ds_bit_spmv(ds_ctx* ctx, const uint64_t* B, int64_t rows, int64_t cols, int64_t stride, int64_t row_first,
                int64_t row_step, const double* x, double* out);
// ---- products of the CGLS matrix of a large game in fixed point (exact integer sums) ----
// Every product starts with ds_vec_quantize: scal[1] (the bit pattern of max |x|, 0 on entry) is found over
// x_all[0..len_all), scal[0] becomes the power of two that scales integer results back, and the vector is written as
// digit planes for the matrix-core product (x_planes[0..planes->cols), if `planes` has rows) and/or as 64-bit
// integers q64[i] = round(x_q[i] * 2^f), i < qlen (if qlen > 0). The product that runs last clears scal[1].
//
// Dense rows on the int8 matrix cores (x split into base-256 digits); out = (addend or 0) + result. A plan fixes
// the launch shape and the scratch of one (rows, cols) shape: ds_bit_spmv_mm_ws_bytes bytes at `ws`, which
// ds_bit_spmv_mm_prepare initialises (on ctx->stream).
struct ds_mm_plan {
  int64_t rows, cols, row_groups, n_chunks, groups, cpg, npad;
  int8_t* D;         // eight digit planes of npad bytes (the last one stays zero)
  int32_t* partial;  // [groups][rows][8] digit sums
};
size_t ds_bit_spmv_mm_ws_bytes(const ds_ctx* ctx, int64_t rows, int64_t cols);
int ds_bit_spmv_mm_prepare(ds_ctx* ctx, int64_t rows, int64_t cols, void* ws, ds_mm_plan* plan);
// with_absmax == 0: the caller's own kernel has left the maximum in scal[1]
int ds_vec_quantize(ds_ctx* ctx, const double* x_all, int64_t len_all, const ds_mm_plan* planes, const double* x_planes,
                    const double* x_q, int64_t qlen, long long* q64, double* scal, int with_absmax = 1);
// out == nullptr: the per-group digit sums are left for the caller's own kernel to add up (ds_mm_sum below)
int ds_bit_spmv_mm_product(ds_ctx* ctx, const ds_mm_plan* plan, const uint64_t* B, int64_t stride, int64_t row_first,
                           int64_t row_step, const double* scal, const double* addend, double* out, int clear_slot);

// Sparse rows as 2-D tiles of (row, column) entries: one list serves both products. Built from the index lists of the
// rows (off = exclusive prefix sums of the row sizes, idx = ascending columns); rows must not hold more than
// max_row_size entries. ws: ds_tile_ws_bytes bytes. The plan keeps `idx`'s memory (the entries end up there) and
// `off` is free after the call.
struct ds_tile_plan {
  int64_t rows, cols, nnz;
  int32_t nrb, ncb, nga, gf, cpg;   // row blocks, column chunks, adjoint row-block groups, forward chunk groups (of cpg)
  int sh_f, sh_a;                   // bits dropped (rounded) from the 2^-54-scaled integers so that the sums fit 63 bits
  int32_t *rb_start, *ga_start, *tile_off;
  uint32_t* ent;
  long long* partial;
};
size_t ds_tile_ws_bytes(const ds_ctx* ctx, int64_t rows, int64_t cols, int64_t nnz);
int ds_tile_build(ds_ctx* ctx, int64_t rows, int64_t cols, int64_t nnz, int64_t max_row_size, const int32_t* off,
                  int32_t* idx, void* ws, ds_tile_plan* plan);
// forward: out[r] = sum of x[c] over the entries of row r (q64 = the 64-bit form of x, cols entries);
// adjoint: out[c] = sum of x[r] over the entries of column c (q64 of rows entries)
// out == nullptr: the per-group partial vectors are left for the caller's own kernel to add up (ds_tile_sum below)
int ds_tile_spmv(ds_ctx* ctx, const ds_tile_plan* plan, int adjoint, const long long* q64, const double* scal, double* out,
                 int clear_slot);

// Where the integer results of one product lie before they are added up, for kernels that consume them directly
// (groups == 0: that part of the matrix is empty).
struct ds_fixed_view {
  const long long* tile_partial;  // [tile_groups][tile_len]
  int64_t tile_len;
  int tile_groups, tile_sh;
  const int32_t* mm_partial;      // [mm_groups][mm_rows][8]
  int64_t mm_rows;
  int mm_groups;
};
static inline ds_fixed_view ds_fixed_view_of(const ds_tile_plan* t, const ds_mm_plan* m, int adjoint) {
  ds_fixed_view v;
  const bool has_t = t && t->rows > 0 && t->nnz > 0, has_m = m && m->rows > 0;
  v.tile_partial = has_t ? t->partial : nullptr;
  v.tile_len = has_t ? (adjoint ? t->cols : t->rows) : 0;
  v.tile_groups = has_t ? (adjoint ? t->nga : t->gf) : 0;
  v.tile_sh = has_t ? (adjoint ? t->sh_a : t->sh_f) : 0;
  v.mm_partial = has_m ? m->partial : nullptr;
  v.mm_rows = has_m ? m->rows : 0;
  v.mm_groups = has_m ? (int)m->groups : 0;
  return v;
}
#ifdef __HIPCC__
// The sums over the groups are exact integers, so they may be split over T lanes in any way: lane `sub` (0 <= sub < T)
// adds the groups sub, sub + T, ... (four loads in flight), the lanes' integers are added, and one rounding ends it.
// tile product, entry i: the groups as two 32-bit halves, so that the total may exceed 63 bits
__device__ __forceinline__ void ds_tile_sum_part(const long long* partial, int64_t len, int groups, int64_t i, int sub, int T,
                                                 long long& hi, long long& lo) {
  int g = sub;
  for (; g + 3 * T < groups; g += 4 * T) {
    const long long* q = partial + (int64_t)g * len + i;
    const int64_t st = (int64_t)T * len;
    const long long p0 = q[0], p1 = q[st], p2 = q[2 * st], p3 = q[3 * st];
    hi += (p0 >> 32) + (p1 >> 32) + (p2 >> 32) + (p3 >> 32);
    lo += (p0 & 0xffffffffll) + (p1 & 0xffffffffll) + (p2 & 0xffffffffll) + (p3 & 0xffffffffll);
  }
  for (; g < groups; g += T) {
    const long long p = partial[(int64_t)g * len + i];
    hi += p >> 32;
    lo += p & 0xffffffffll;
  }
}
// ... times 2^sh
__device__ __forceinline__ double ds_tile_sum_finish(long long hi, long long lo, int sh) {
  return ((double)hi * 4294967296.0 + (double)lo) * (double)(1ll << sh);
}
__device__ __forceinline__ double ds_tile_sum(const long long* partial, int64_t len, int groups, int sh, int64_t i) {
  long long hi = 0, lo = 0;
  ds_tile_sum_part(partial, len, groups, i, 0, 1, hi, lo);
  return ds_tile_sum_finish(hi, lo, sh);
}
// matrix-core product, row r: S[d] = sum over the groups of digit sum d; the result is sum_d 256^d S[d]
__device__ __forceinline__ void ds_mm_sum_part(const int32_t* partial, int64_t rows, int groups, int64_t r, int sub, int T,
                                               long long S[7]) {
  int g = sub;
  for (; g + T < groups; g += 2 * T) {
    const int4* p = (const int4*)(partial + ((int64_t)g * rows + r) * 8);
    const int4* q = (const int4*)(partial + ((int64_t)(g + T) * rows + r) * 8);
    const int4 u = p[0], w = p[1], u2 = q[0], w2 = q[1];
    S[0] += (long long)u.x + u2.x;
    S[1] += (long long)u.y + u2.y;
    S[2] += (long long)u.z + u2.z;
    S[3] += (long long)u.w + u2.w;
    S[4] += (long long)w.x + w2.x;
    S[5] += (long long)w.y + w2.y;
    S[6] += (long long)w.z + w2.z;
  }
  for (; g < groups; g += T) {
    const int4* p = (const int4*)(partial + ((int64_t)g * rows + r) * 8);
    const int4 u = p[0], w = p[1];
    S[0] += u.x;
    S[1] += u.y;
    S[2] += u.z;
    S[3] += u.w;
    S[4] += w.x;
    S[5] += w.y;
    S[6] += w.z;
  }
}
__device__ __forceinline__ double ds_mm_sum_finish(const long long S[7]) {
  const long long hi = ((S[6] * 256 + S[5]) * 256 + S[4]) * 256 + S[3];
  const long long lo = (S[2] * 256 + S[1]) * 256 + S[0];
  return (double)hi * 16777216.0 + (double)lo;
}
__device__ __forceinline__ double ds_mm_sum(const int32_t* partial, int64_t rows, int groups, int64_t r) {
  long long S[7] = {0, 0, 0, 0, 0, 0, 0};
  ds_mm_sum_part(partial, rows, groups, r, 0, 1, S);
  return ds_mm_sum_finish(S);
}
#endif

// index lists of the set bits of rows (off = exclusive prefix sums of the row sizes)
int ds_rows_to_csr(ds_ctx* ctx, const uint64_t* B, int64_t rows, int64_t cols, int64_t stride, int64_t row_first,
                   int64_t row_step, const int32_t* off, int32_t* idx);
