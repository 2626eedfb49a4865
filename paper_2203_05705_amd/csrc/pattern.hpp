// Pattern generation entry used by the GEMM entry points.
#pragma once
#include "common.hpp"

namespace ard {
// Enqueue mask / kept-list / offsets generation for a ROW or TILE pattern
// (arguments as ard_pattern_gen, already validated).
int32_t pattern_gen_launch(const ard_pattern* pat, int32_t rows, int32_t cols, uint8_t* d_mask, int32_t* d_keep,
                           int32_t* d_count, int32_t* d_rowptr, int32_t* d_colptr, int32_t* d_csc_rows,
                           hipStream_t stream);
int32_t fill_matrix(int32_t dtype, void* p, long n, float beta, hipStream_t stream);
}  // namespace ard
