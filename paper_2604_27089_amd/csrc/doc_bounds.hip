// Per-row document window for packed variable-length batches: for every row i,
// row_lo[i] = first row of its document and row_hi[i] = one past its last row.
// Values are clamped so that row_lo[i] <= i < row_hi[i] <= T whatever the
// contents of cu_seqlens: a malformed array gives wrong masks, never a wild
// address.
#include "sp_common.h"

namespace {

__global__ __launch_bounds__(256) void doc_bounds_kernel(const int32_t* __restrict__ cu,
                                                        int32_t n_docs, int32_t T,
                                                        int32_t* __restrict__ row_lo,
                                                        int32_t* __restrict__ row_hi) {
    const int32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= T) return;
    // last t in [0, n_docs) with cu[t] <= i  (empty documents share a start; the
    // last one with that start is the one that owns the row)
    int32_t lo = 0, hi = n_docs;  // invariant: answer in [lo, hi)
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (cu[mid] <= i) lo = mid; else hi = mid;
    }
    int32_t a = cu[lo], b = cu[lo + 1];
    a = a < 0 ? 0 : (a > i ? i : a);
    b = b > T ? T : (b < i + 1 ? i + 1 : b);
    row_lo[i] = a;
    row_hi[i] = b;
}

}  // namespace

namespace sp {

sp_status launch_doc_bounds(const int32_t* cu_seqlens, int32_t n_docs, int32_t T, int32_t* row_lo,
                            int32_t* row_hi, hipStream_t st) {
    if (T <= 0) return SP_OK;
    hipLaunchKernelGGL(doc_bounds_kernel, dim3((T + 255) / 256), dim3(256), 0, st, cu_seqlens,
                       n_docs, T, row_lo, row_hi);
    return launch_status();
}

}  // namespace sp
