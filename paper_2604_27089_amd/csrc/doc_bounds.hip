// Per-row document window for packed variable-length batches: for every row i,
// row_lo[i] = first row of its document and row_hi[i] = one past its last row.
// Values are clamped so that row_lo[i] <= i < row_hi[i] <= T whatever the
// contents of cu_seqlens: a malformed array gives wrong masks, never a wild
// address.
//
// Also here: the order in which the attention kernels' workgroups take their
// 256-row (or 256-key) tiles.  With documents of mixed lengths the work of a tile
// is not a function of its position (a query tile walks the keys of its own
// document only), and with a few workgroups per compute unit the kernel ends
// when the unluckiest unit does: tiles are handed out longest first, which is
// what the dense kernels' "last query tile first" order amounts to.
#include "sp_common.h"

namespace {

using namespace sp;

// Besides the per-row windows, the first and the last row of every 256-row tile leave the tile's work for the
// ordering below (when `work_q` is not null): a query tile (forward, dQ) walks the 64-key tiles from the start
// of its first row's document to its last row; a key tile (dK/dV) walks the 32-row tiles from its first key
// to the end of its last key's document.
__global__ __launch_bounds__(256) void doc_bounds_kernel(const int32_t* __restrict__ cu,
                                                        int32_t n_docs, int32_t T,
                                                        int32_t* __restrict__ row_lo,
                                                        int32_t* __restrict__ row_hi,
                                                        int32_t* __restrict__ work_q,
                                                        int32_t* __restrict__ work_k) {
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
    if (work_q) {
        static_assert(kOrderTile == 256, "one block of this kernel is one tile");
        const int32_t first = blockIdx.x * kOrderTile;
        const int32_t last = first + kOrderTile - 1 < T ? first + kOrderTile - 1 : T - 1;
        if (i == first) work_q[blockIdx.x] = last / 64 + 1 - a / 64;
        if (i == last) work_k[blockIdx.x] = (b + 31) / 32 - first / 32;
    }
}

// order[r] = the tile of rank r: more work first; among equals the later query tile, resp. the earlier key
// tile, first (the dense kernels' orders).  One workgroup per tile counts the tiles that precede it under a
// strict total order, so the ranks are a permutation of 0 .. n_tiles-1 and every entry of both arrays is
// written exactly once.
__global__ __launch_bounds__(256) void tile_rank_kernel(const int32_t* __restrict__ work_q,
                                                       const int32_t* __restrict__ work_k, int32_t n_tiles,
                                                       int32_t* __restrict__ order_q,
                                                       int32_t* __restrict__ order_k) {
    __shared__ int32_t part[2][4];
    const int32_t t = blockIdx.x;
    const int32_t wq = work_q[t], wk = work_k[t];
    int32_t rq = 0, rk = 0;
    for (int32_t u = threadIdx.x; u < n_tiles; u += 256) {
        const int32_t oq = work_q[u], ok = work_k[u];
        rq += (oq > wq || (oq == wq && u > t)) ? 1 : 0;
        rk += (ok > wk || (ok == wk && u < t)) ? 1 : 0;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        rq += __shfl_xor(rq, off, 64);
        rk += __shfl_xor(rk, off, 64);
    }
    if ((threadIdx.x & 63) == 0) { part[0][threadIdx.x >> 6] = rq; part[1][threadIdx.x >> 6] = rk; }
    __syncthreads();
    if (threadIdx.x == 0) {
        order_q[part[0][0] + part[0][1] + part[0][2] + part[0][3]] = t;
        order_k[part[1][0] + part[1][1] + part[1][2] + part[1][3]] = t;
    }
}

// Debug aid: does a cu_seqlens array describe T rows?  One workgroup scans the n_docs + 1 entries and writes a
// bit mask to *flag (0 = well formed): 1 cu[0] != 0, 2 some cu[t+1] < cu[t], 4 cu[n_docs] != T.  The attention
// kernels never depend on it: they clamp what they read.
__global__ __launch_bounds__(256) void check_cu_seqlens_kernel(const int32_t* __restrict__ cu, int32_t n_docs, int32_t T,
                                                              int32_t* __restrict__ flag) {
    __shared__ int32_t part[4];
    int32_t bad = 0;
    for (int32_t t = threadIdx.x; t <= n_docs; t += 256) {
        const int32_t c = cu[t];
        if (t == 0 && c != 0) bad |= 1;
        if (t == n_docs && c != T) bad |= 4;
        if (t < n_docs && cu[t + 1] < c) bad |= 2;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) bad |= __shfl_xor(bad, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = bad;
    __syncthreads();
    if (threadIdx.x == 0) *flag = part[0] | part[1] | part[2] | part[3];
}

}  // namespace

namespace sp {

sp_status launch_check_cu_seqlens(const int32_t* cu_seqlens, int32_t n_docs, int32_t T, int32_t* flag, hipStream_t st) {
    hipLaunchKernelGGL(check_cu_seqlens_kernel, dim3(1), dim3(256), 0, st, cu_seqlens, n_docs, T, flag);
    return launch_status();
}

sp_status launch_doc_bounds(const int32_t* cu_seqlens, int32_t n_docs, int32_t T, int32_t* row_lo,
                            int32_t* row_hi, int32_t* work, int32_t* order_q, int32_t* order_k, hipStream_t st) {
    if (T <= 0) return SP_OK;
    const int32_t n = order_tiles(T);  // = the grid of the first kernel
    hipLaunchKernelGGL(doc_bounds_kernel, dim3(n), dim3(256), 0, st, cu_seqlens, n_docs, T, row_lo, row_hi,
                       work, work ? work + n : nullptr);
    if (launch_status() != SP_OK) return SP_ERR_LAUNCH;
    if (!work) return SP_OK;
    hipLaunchKernelGGL(tile_rank_kernel, dim3(n), dim3(256), 0, st, work, work + n, n, order_q, order_k);
    return launch_status();
}

}  // namespace sp
