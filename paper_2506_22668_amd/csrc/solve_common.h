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
// out[i] = sum of x[j] over the set bits j < cols of row (row_first + i*row_step) of B, i < rows (fp64)
int ds_bit_spmv(ds_ctx* ctx, const uint64_t* B, int64_t rows, int64_t cols, int64_t stride, int64_t row_first,
                int64_t row_step, const double* x, double* out);
// The same product for dense rows on the int8 matrix cores (x split into base-256 digits: exact integer sums);
// out = (addend or 0) + result. A plan fixes the launch shape and the scratch of one (rows, cols) shape:
// ds_bit_spmv_mm_ws_bytes bytes at `ws`, which ds_bit_spmv_mm_prepare initialises (on ctx->stream).
struct ds_mm_plan {
  int64_t rows, cols, row_groups, n_chunks, groups, cpg, npad;
  double* scal;      // [0] scale of the current product, [1] bit pattern of max |x| (cleared by every product)
  int8_t* D;         // eight digit planes of npad bytes (the last one stays zero)
  int32_t* partial;  // [groups][rows][8] digit sums
};
size_t ds_bit_spmv_mm_ws_bytes(const ds_ctx* ctx, int64_t rows, int64_t cols);
int ds_bit_spmv_mm_prepare(ds_ctx* ctx, int64_t rows, int64_t cols, void* ws, ds_mm_plan* plan);
// A product is two calls: the digits of x (two small kernels), then the product proper.
// addend_ready: optional event the final summation waits for (an addend produced on another stream)
int ds_bit_spmv_mm_digits(ds_ctx* ctx, const ds_mm_plan* plan, const double* x);
int ds_bit_spmv_mm_product(ds_ctx* ctx, const ds_mm_plan* plan, const uint64_t* B, int64_t stride, int64_t row_first,
                           int64_t row_step, const double* addend, double* out, hipEvent_t addend_ready = nullptr);
// index lists of the set bits of rows (off = exclusive prefix sums of the row sizes), and the gather-sum over them
int ds_rows_to_csr(ds_ctx* ctx, const uint64_t* B, int64_t rows, int64_t cols, int64_t stride, int64_t row_first,
                   int64_t row_step, const int32_t* off, int32_t* idx);
int ds_csr_gather(ds_ctx* ctx, const int32_t* off, const int32_t* idx, int64_t rows, const double* x, double* out);
