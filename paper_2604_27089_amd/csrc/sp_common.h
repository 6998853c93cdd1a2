// Shared host-side declarations of the C-ABI layer (validation helpers and the
// kernel launchers implemented in the .hip files).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sp_hotpath.h"

namespace sp {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline sp_status launch_status() {
    return hipGetLastError() == hipSuccess ? SP_OK : SP_ERR_LAUNCH;
}

// Where row r (0 <= r < S) of an attention-side [S, H, D] tensor lives, in elements from the start of
// its batch entry (the head offset h*D comes on top).  Two layouts are served by the same kernels:
//   attention-side  [S, H, D]        : r * H*D
//   sequence-side   [S_l, P*H, D]    : (r % S_l) * P*H*D + (r / S_l) * H*D
// the second being the tensor whose pack (seq -> head re-layout) is the first: reading through this map
// folds the pack into the attention kernels' loads and the unpack into their stores.  S_l is a power
// of two there (mask/shift); the attention-side case uses shift 31, so r >> shift is 0 for every row.
// A batch entry spans S*H*D elements in both layouts.
struct RowMap {
    uint32_t mask;          // S_l - 1, or 0x7fffffff
    int32_t shift;          // log2(S_l), or 31
    uint32_t row_stride;    // elements between consecutive rows of a chunk
    uint32_t chunk_stride;  // elements between chunk p and chunk p+1 (H*D, or 0)
    __host__ __device__ size_t off(int32_t r) const {
        return (size_t)((uint32_t)r & mask) * row_stride + (size_t)((uint32_t)r >> shift) * chunk_stride;
    }
    static RowMap attention_side(int32_t H, int32_t D) { return RowMap{0x7fffffffu, 31, (uint32_t)(H * D), 0u}; }
    static RowMap sequence_side(int32_t S_l_log2, int32_t H, int32_t D, int32_t P) {
        return RowMap{(1u << S_l_log2) - 1u, S_l_log2, (uint32_t)(P * H * D), (uint32_t)(H * D)};
    }
};

// One attention problem as the kernels see it.  Dense calls are B independent
// sequences of S rows; packed-document calls are B = 1, S = T rows with a
// per-row visibility window taken from `row_lo` / `row_hi`.  In general the S
// query rows face Skv keys and row i sees keys j <= i + off (one step of a ring
// schedule); every key must be seen by some row (Skv <= S + off, off >= 0).
// Causal attention over one sequence is Skv = S, off = 0.
struct AttnArgs {
    const void* q; const void* k; const void* v;   // bf16
    void* o; float* lse;                           // fwd outputs (bwd: inputs)
    const void* dO; void* dq; void* dk; void* dv;  // bwd only
    float* delta;                                  // bwd workspace, [B, Hq, S] fp32
    float* aux;                                    // bwd workspace, [B*Hq, S_pad/32, 2, 32] fp32: per 32-row
                                                   // tile, 32 x -LSE/scale then 32 x -Delta
    int32_t S_pad;                                 // rows per head in aux (S rounded up to 64, plus 64)
    const int32_t* row_lo;  // varlen: first row of the row's document, [S]; null if dense
    const int32_t* row_hi;  // varlen: one past the last row of the row's document, [S]
    const int32_t* order_q; // varlen: query tiles (256 rows) in the order workgroups take them; null = last first
    const int32_t* order_k; // varlen: key tiles (256 keys) likewise; null = first first
    int32_t B, S, Hq, Hkv, D;
    int32_t Skv, off;       // keys per sequence; causal offset
    RowMap qmap, kvmap;     // layout of q, o, dO, dq and of k, v, dk, dv
    float scale;            // softmax scale (already defaulted)
    int32_t stages;         // bwd: bit mask of SP_BWD_STAGE_*
    int32_t dkdv_splits;    // bwd: workgroups that share one key tile of the dK/dV kernel (dkdv_split_count)
    float* dkdv_part;       // bwd workspace: their fp32 partial sums (null when dkdv_splits == 1)
};

sp_status launch_relayout(const void* in, void* out, int64_t B, int64_t S_l, int64_t H, int64_t D,
                          int32_t P, int32_t elem_bytes, bool to_head, hipStream_t st);
// Longest-first tile orders for packed documents (doc_bounds.hip).  All three attention kernels use tiles
// of kOrderTile rows resp. keys per workgroup.  Above kMaxOrderTiles tiles the quadratic ranking is not
// worth its time and callers pass null orders.
constexpr int32_t kOrderTile = 256;
constexpr int32_t kMaxOrderTiles = 16384;
inline int32_t order_tiles(int64_t T) { return (int32_t)((T + kOrderTile - 1) / kOrderTile); }
// Per-row document windows, and (if `work` is not null) the tile orders: `work` is scratch of
// 2*order_tiles(T) int32, `order_q`, `order_k` receive order_tiles(T) int32 each.
sp_status launch_doc_bounds(const int32_t* cu_seqlens, int32_t n_docs, int32_t T, int32_t* row_lo,
                            int32_t* row_hi, int32_t* work, int32_t* order_q, int32_t* order_k, hipStream_t st);
// Debug aid: writes 0 to *flag if cu_seqlens is well formed for T rows, else a bit mask (doc_bounds.hip).
sp_status launch_check_cu_seqlens(const int32_t* cu_seqlens, int32_t n_docs, int32_t T, int32_t* flag, hipStream_t st);
// Grid of the forward and dQ kernels: x = head + Hq * batch, (y, z) = rank of the query tile in the order the
// tiles are taken (rank = y + kRankY * z).  Workgroups are dispatched x first, so all heads and batch entries
// of the longest tile go out before any shorter tile (a batch-major order would end with the long tiles of
// the last batch entry).
constexpr uint32_t kRankY = 32768;
inline dim3 tile_rank_grid(int32_t Hq, int32_t B, int32_t n_tiles) {
    return dim3((uint32_t)Hq * (uint32_t)B, (uint32_t)n_tiles < kRankY ? (uint32_t)n_tiles : kRankY,
                ((uint32_t)n_tiles + kRankY - 1) / kRankY);
}
sp_status launch_attn_fwd(const AttnArgs& a, hipStream_t st);
sp_status launch_attn_bwd(const AttnArgs& a, hipStream_t st);
sp_status launch_attn_bwd_dkdv(const AttnArgs& a, hipStream_t st);
sp_status launch_attn_bwd_dq(const AttnArgs& a, hipStream_t st);
sp_status launch_attn_merge(float* o_acc, float* lse_acc, const void* o_blk, const float* lse_blk, void* o_out,
                            int64_t B, int64_t S, int32_t Hq, int32_t D, hipStream_t st);

// How many workgroups share one 256-key tile of the dK/dV kernel.  A key tile's work is every row from
// its diagonal to the end of the sequence (or document), for every query head of the group: with one KV
// head that is one workgroup per 256 keys, far too few to fill and balance 256 compute units below a
// few hundred thousand rows (at 32K rows: 128 workgroups, the longest doing 1/64 of all the work).  The
// (head, row tile) steps of a key tile are therefore cut into this many contiguous chunks, one workgroup
// each, whose fp32 partial sums a second kernel adds in a fixed order (measured: 4.36 -> 1.65 ms at 32K
// rows, 10.1 -> 6.3 ms at 64K, 25.3 -> 24.7 ms at 128K).
// A workgroup of this kernel costs about 45 us beyond its steps (loading its keys and values, the pipeline
// prologue, writing 256 KB of partial sums), a step about 1.5 us, and one compute unit holds one workgroup:
// n chunks per tile cost (tiles * n / 256) * 45 us of overhead and leave a longest chunk of steps_first / n
// steps, a fraction of which is exposed at the end.  The sum is smallest near n = sqrt(2.1 * steps_first /
// tiles) (the constant fitted to sequences of 1K to 128K rows, dense and packed); at most 8 chunks, and no
// more than about 2048 workgroups.  `longest` = the longest sequence in the call when the caller knows it
// (packed documents: the max_seqlen hint), else S.  The count depends on these extents only, so packed
// documents and dense calls of equal extents agree bitwise.
inline int32_t dkdv_split_count(int64_t B, int64_t S, int64_t Skv, int32_t Hq, int32_t Hkv, int64_t longest = 0) {
    if (B <= 0 || S <= 0 || Skv <= 0 || Hkv <= 0) return 1;
    if (longest <= 0 || longest > S) longest = S;
    const int64_t tiles = (Skv + 255) / 256 * Hkv * B;
    const int64_t steps_first = (longest + 31) / 32 * (Hq / Hkv);  // steps of the longest key tile
    int64_t n = 1;
    while (n < 8 && (2 * n + 1) * (2 * n + 1) * tiles * 10 <= 4 * 21 * steps_first) ++n;  // n <= sqrt(2.1 x) + 0.5
    // Several sequences are dispatched batch entry fastest, longest tiles of every sequence first: there two
    // workgroups per compute unit balance better than one even where the rule above says one chunk (256 tiles:
    // 32 x 2048 rows 392 -> 336 us, 64 x 1024 rows 230 -> 220 us).
    if (B > 1 && n * tiles < 512) n = (512 + tiles - 1) / tiles < 8 ? (512 + tiles - 1) / tiles : 8;
    const int64_t cap = (2048 + tiles - 1) / tiles;
    if (n > cap) n = cap;
    return n < 1 ? 1 : (int32_t)n;
}
inline size_t dkdv_part_bytes(int64_t B, int64_t Skv, int32_t Hkv, int32_t D, int32_t nsplit) {
    return nsplit > 1 ? (size_t)2 * nsplit * B * Skv * Hkv * D * sizeof(float) : 0;
}

// pointwise operators outside attention (pointwise.hip)
sp_status launch_rmsnorm_fwd(const void* x, const void* w, void* y, float* rstd, int64_t T, int32_t C, float eps,
                             hipStream_t st);
sp_status launch_rmsnorm_bwd(const void* x, const void* w, const float* rstd, const void* dy, void* dx, void* dw,
                             float* part, int64_t T, int32_t C, hipStream_t st);
int32_t rmsnorm_bwd_groups(int64_t T);  // partial rows of dw the backward writes to its workspace
sp_status launch_rope(const void* x, const float* cs, const float* sn, void* out, int64_t T, int32_t H, int32_t D,
                      bool conjugate, hipStream_t st);
sp_status launch_swiglu_fwd(const void* g, const void* u, void* y, int64_t n, hipStream_t st);
sp_status launch_swiglu_bwd(const void* g, const void* u, const void* dy, void* dg, void* du, int64_t n, hipStream_t st);

// row pitch of the per-row backward scalars
inline int32_t aux_pitch(int64_t S) { return (int32_t)((S + 63) / 64 * 64 + 64); }

}  // namespace sp
