// Internal entry points shared between the translation units of the library.
#pragma once

#include "lshe_common.h"

namespace lshe {

// Hash n_rows vectors addressed as (segment, index) pairs; see hash_rows_kernel.  out_stride < 0:
// the call covers whole segments and the codes go to consecutive rows.
int hash_rows(const Dims &m, const void *R_dev, const void *X, int64_t n_rows, int64_t seg_len,
              int64_t seg_stride, int64_t seg_off, uint32_t *codes, hipStream_t st,
              int64_t out_stride = -1, int64_t out_off = 0);

// L2-norm policy: codes[f] = bit pattern of the squared norm of row f of X (rows contiguous).
int norm_rows(const Dims &m, const void *X, int64_t n_rows, uint32_t *codes, hipStream_t st);

}  // namespace lshe
