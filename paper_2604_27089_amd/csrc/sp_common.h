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

// One attention problem as the kernels see it.  Dense calls are B independent
// sequences of S rows; packed-document calls are B = 1, S = T rows with a
// per-row visibility window taken from `row_lo` / `row_hi`.
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
    int32_t B, S, Hq, Hkv, D;
    float scale;            // softmax scale (already defaulted)
    int32_t stages;         // bwd: bit mask of SP_BWD_STAGE_*
};

sp_status launch_relayout(const void* in, void* out, int64_t B, int64_t S_l, int64_t H, int64_t D,
                          int32_t P, int32_t elem_bytes, bool to_head, hipStream_t st);
sp_status launch_doc_bounds(const int32_t* cu_seqlens, int32_t n_docs, int32_t T, int32_t* row_lo,
                            int32_t* row_hi, hipStream_t st);
sp_status launch_attn_fwd(const AttnArgs& a, hipStream_t st);
sp_status launch_attn_bwd(const AttnArgs& a, hipStream_t st);
sp_status launch_attn_bwd_dkdv(const AttnArgs& a, hipStream_t st);
sp_status launch_attn_bwd_dq(const AttnArgs& a, hipStream_t st);

// row pitch of the per-row backward scalars
inline int32_t aux_pitch(int64_t S) { return (int32_t)((S + 63) / 64 * 64 + 64); }

}  // namespace sp
