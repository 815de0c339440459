// Launchers of the per-wavefront gather kernel, one set per operand format,
// compiled in translation units of their own so that the library builds in
// parallel.  ydtype has been checked by the caller.
#pragma once
#include <hip/hip_runtime.h>

#include "gather_kernel.hip"
#include "shflbw_internal.h"

namespace shflbw {

int run_gather_f16(const shflbw_matrix* A, const GeomLinear<true>& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_f16(const shflbw_matrix* A, const GeomLinearBuf& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_f16(const shflbw_matrix* A, const GeomLinear<false>& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_f16(const shflbw_matrix* A, const GeomConv& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_f16(const shflbw_matrix* A, const GeomBatchedBuf& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_f16(const shflbw_matrix* A, const GeomBatchedBuf4& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_bf16(const shflbw_matrix* A, const GeomLinear<true>& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_bf16(const shflbw_matrix* A, const GeomLinearBuf& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_bf16(const shflbw_matrix* A, const GeomLinear<false>& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_bf16(const shflbw_matrix* A, const GeomConv& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_bf16(const shflbw_matrix* A, const GeomBatchedBuf& g, long N, shflbw_dtype ydtype, hipStream_t stream);
int run_gather_bf16(const shflbw_matrix* A, const GeomBatchedBuf4& g, long N, shflbw_dtype ydtype, hipStream_t stream);

}  // namespace shflbw
