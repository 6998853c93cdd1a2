// C-ABI entry points: argument validation on the host, then kernel launches on
// the caller's stream.  Nothing here allocates, frees or synchronises.  The only
// state kept between calls is the per-device address of one static scratch array.
#include <math.h>

#include <mutex>

#include "sp_common.h"

namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

sp_status check_relayout(const void* in, void* out, int64_t B, int64_t S_l, int64_t H, int64_t D,
                         int32_t P, int32_t elem_bytes) {
    if (B < 0 || S_l < 0 || H < 0 || D < 0 || P <= 0) return SP_ERR_SHAPE;
    if (H % P != 0) return SP_ERR_SHAPE;
    if (elem_bytes != 2 && elem_bytes != 4) return SP_ERR_UNSUPPORTED;
    if ((D * elem_bytes) % 16 != 0) return SP_ERR_UNSUPPORTED;
    if (B == 0 || S_l == 0 || H == 0 || D == 0) return SP_OK;
    if (!in || !out) return SP_ERR_NULL;
    if (!sp::aligned16(in) || !sp::aligned16(out)) return SP_ERR_ALIGN;
    return SP_OK;
}

sp_status check_attn_shape(int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D) {
    if (B < 0 || S < 0 || Hq < 0 || Hkv < 0) return SP_ERR_SHAPE;
    if (Hq == 0 || Hkv == 0) return (Hq == 0 && Hkv == 0) ? SP_OK : SP_ERR_SHAPE;
    if (Hq % Hkv != 0) return SP_ERR_SHAPE;
    if (D != 64 && D != 128) return SP_ERR_UNSUPPORTED;
    if (S >= (int64_t)1 << 31 || B >= (int64_t)1 << 16 || B * S >= (int64_t)1 << 31) return SP_ERR_SHAPE;
    return SP_OK;
}

inline float resolve_scale(float s, int32_t D) { return s > 0.f ? s : 1.0f / sqrtf((float)D); }

inline void attention_side_maps(sp::AttnArgs& a) {
    a.qmap = sp::RowMap::attention_side(a.Hq, a.D);
    a.kvmap = sp::RowMap::attention_side(a.Hkv, a.D);
}

// sequence-side calls: S_l must be a power of two and a multiple of the largest tile (256 rows), so that
// no tile of any kernel straddles two peers' chunks; returns log2(S_l) or -1
inline int32_t seq_chunk_log2(int64_t S_l) {
    if (S_l < 256 || (S_l & (S_l - 1)) != 0 || S_l >= ((int64_t)1 << 31)) return -1;
    int32_t l = 0;
    while (((int64_t)1 << l) < S_l) ++l;
    return l;
}

// Workspace layout: [delta fp32 B*Hq*S] [per-row seeds fp32 2*B*Hq*S_pad: per 32-row tile, 32 x -LSE/scale
// then 32 x -Delta] (bwd only)
// [row_lo int32 T] [row_hi int32 T] [tile work 2n int32, query-tile order n, key-tile order n; n = ceil(T/256)]
// (varlen only; the order block is absent above kMaxOrderTiles tiles)
// [dK/dV partial sums fp32 2*nsplit*B*S*Hkv*D] (bwd only, when the dK/dV kernel splits its key tiles),
// each part rounded up to 256 bytes.
size_t delta_bytes(int64_t T, int32_t Hq) { return align_up((size_t)T * (size_t)Hq * sizeof(float), 256); }
size_t bounds_bytes(int64_t T) { return align_up((size_t)T * sizeof(int32_t), 256); }
size_t order_bytes(int64_t T) {
    const int64_t n = sp::order_tiles(T);
    return n <= sp::kMaxOrderTiles ? align_up((size_t)4 * n * sizeof(int32_t), 256) : 0;
}
size_t aux_bytes(int64_t B, int64_t S, int32_t Hq) {
    return align_up((size_t)B * (size_t)Hq * (size_t)sp::aux_pitch(S) * sizeof(float), 256);
}
// common tail of the dense forward entry points
sp_status run_dense_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B, int64_t Sq,
                        int64_t Skv, int64_t off, int32_t Hq, int32_t Hkv, int32_t D, const sp::RowMap& qmap,
                        const sp::RowMap& kvmap, float softmax_scale, void* hip_stream) {
    if (!q || !k || !v || !o || !lse) return SP_ERR_NULL;
    if (!sp::aligned16(q) || !sp::aligned16(k) || !sp::aligned16(v) || !sp::aligned16(o) ||
        !sp::aligned16(lse))
        return SP_ERR_ALIGN;
    sp::AttnArgs a{};
    a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
    a.B = (int32_t)B; a.S = (int32_t)Sq; a.Hq = Hq; a.Hkv = Hkv; a.D = D;
    a.Skv = (int32_t)Skv; a.off = (int32_t)off;
    a.qmap = qmap; a.kvmap = kvmap;
    a.scale = resolve_scale(softmax_scale, D);
    return sp::launch_attn_fwd(a, (hipStream_t)hip_stream);
}

// The dense backward entry points differ in extents, causal offset and row maps only; this is their common
// tail: pointer checks, carving the workspace ([delta][per-row seeds][dK/dV partial sums]), launch.
struct BwdBuffers {
    const void* q; const void* k; const void* v; const void* o; const float* lse; const void* dO;
    void* dq; void* dk; void* dv; void* workspace; size_t workspace_bytes;
};
size_t dense_bwd_bytes(int64_t B, int64_t Sq, int64_t Skv, int32_t Hq, int32_t Hkv, int32_t D) {
    size_t n = delta_bytes(B * Sq, Hq) + 2 * aux_bytes(B, Sq, Hq);
    n += align_up(sp::dkdv_part_bytes(B, Skv, Hkv, D, sp::dkdv_split_count(B, Sq, Skv, Hq, Hkv)), 256);
    return n < 256 ? 256 : n;
}
sp_status run_dense_bwd(const BwdBuffers& t, int64_t B, int64_t Sq, int64_t Skv, int64_t off, int32_t Hq,
                        int32_t Hkv, int32_t D, const sp::RowMap& qmap, const sp::RowMap& kvmap,
                        float softmax_scale, int32_t stages, void* hip_stream) {
    if (stages <= 0 || (stages & ~SP_BWD_STAGE_ALL) != 0) return SP_ERR_SHAPE;
    if (!t.q || !t.k || !t.v || !t.o || !t.lse || !t.dO || !t.dq || !t.dk || !t.dv || !t.workspace) return SP_ERR_NULL;
    const void* ptrs[] = {t.q, t.k, t.v, t.o, t.lse, t.dO, t.dq, t.dk, t.dv, t.workspace};
    for (const void* p : ptrs)
        if (!sp::aligned16(p)) return SP_ERR_ALIGN;
    if (t.workspace_bytes < dense_bwd_bytes(B, Sq, Skv, Hq, Hkv, D)) return SP_ERR_WORKSPACE;
    sp::AttnArgs a{};
    a.q = t.q; a.k = t.k; a.v = t.v; a.o = const_cast<void*>(t.o); a.lse = const_cast<float*>(t.lse);
    a.dO = t.dO; a.dq = t.dq; a.dk = t.dk; a.dv = t.dv;
    a.delta = (float*)t.workspace;
    a.aux = (float*)((char*)t.workspace + delta_bytes(B * Sq, Hq));
    a.S_pad = sp::aux_pitch(Sq);
    a.B = (int32_t)B; a.S = (int32_t)Sq; a.Hq = Hq; a.Hkv = Hkv; a.D = D;
    a.Skv = (int32_t)Skv; a.off = (int32_t)off;
    a.qmap = qmap; a.kvmap = kvmap;
    a.scale = resolve_scale(softmax_scale, D);
    a.stages = stages;
    a.dkdv_splits = sp::dkdv_split_count(B, Sq, Skv, Hq, Hkv);
    a.dkdv_part = a.dkdv_splits > 1 ? (float*)((char*)a.aux + 2 * aux_bytes(B, Sq, Hq)) : nullptr;
    return sp::launch_attn_bwd(a, (hipStream_t)hip_stream);
}

// per-row document windows and, when the batch is small enough to have an order block (at `blk`), the
// longest-first tile orders
sp_status make_bounds(sp::AttnArgs& a, const int32_t* cu_seqlens, int32_t n_docs, int64_t T, int32_t* row_lo,
                      int32_t* row_hi, void* blk, hipStream_t s) {
    a.row_lo = row_lo; a.row_hi = row_hi;
    if (order_bytes(T) == 0) return sp::launch_doc_bounds(cu_seqlens, n_docs, (int32_t)T, row_lo, row_hi, nullptr, nullptr, nullptr, s);
    const int32_t n = sp::order_tiles(T);
    int32_t* w = (int32_t*)blk;
    a.order_q = w + 2 * n;
    a.order_k = w + 3 * n;
    return sp::launch_doc_bounds(cu_seqlens, n_docs, (int32_t)T, row_lo, row_hi, w, w + 2 * n, w + 3 * n, s);
}

}  // namespace

extern "C" {

const char* sp_status_str(sp_status s) {
    switch (s) {
        case SP_OK: return "SP_OK";
        case SP_ERR_NULL: return "SP_ERR_NULL: a required pointer is NULL";
        case SP_ERR_SHAPE: return "SP_ERR_SHAPE: extents are negative, too large or do not divide";
        case SP_ERR_UNSUPPORTED: return "SP_ERR_UNSUPPORTED: head dim or element size not supported";
        case SP_ERR_WORKSPACE: return "SP_ERR_WORKSPACE: workspace too small";
        case SP_ERR_ALIGN: return "SP_ERR_ALIGN: pointer not 16-byte aligned";
        case SP_ERR_LAUNCH: return "SP_ERR_LAUNCH: HIP launch failed";
    }
    return "SP_ERR_?: unknown status";
}

int32_t sp_abi_version(void) { return 4; }

sp_status sp_pack_seq_to_head(const void* in, void* out, int64_t B, int64_t S_l, int64_t H,
                              int64_t D, int32_t P, int32_t elem_bytes, void* hip_stream) {
    sp_status st = check_relayout(in, out, B, S_l, H, D, P, elem_bytes);
    if (st != SP_OK || B == 0 || S_l == 0 || H == 0 || D == 0) return st;
    return sp::launch_relayout(in, out, B, S_l, H, D, P, elem_bytes, true, (hipStream_t)hip_stream);
}

sp_status sp_unpack_head_to_seq(const void* in, void* out, int64_t B, int64_t S_l, int64_t H,
                                int64_t D, int32_t P, int32_t elem_bytes, void* hip_stream) {
    sp_status st = check_relayout(in, out, B, S_l, H, D, P, elem_bytes);
    if (st != SP_OK || B == 0 || S_l == 0 || H == 0 || D == 0) return st;
    return sp::launch_relayout(in, out, B, S_l, H, D, P, elem_bytes, false, (hipStream_t)hip_stream);
}

size_t sp_attn_bwd_workspace_bytes(int64_t B, int64_t S_or_T, int32_t Hq, int32_t Hkv, int32_t D,
                                   int32_t n_docs) {
    if (n_docs < 0 || B <= 0) return 0;
    if (check_attn_shape(n_docs > 0 ? 1 : B, S_or_T, Hq, Hkv, D) != SP_OK || Hq == 0) return 0;
    if (n_docs == 0) return dense_bwd_bytes(B, S_or_T, S_or_T, Hq, Hkv, D);
    // packed documents: one sequence of T rows, with the windows and tile orders between the seeds and the
    // partial sums (sized for the largest work split, i.e. without a max_seqlen hint)
    const int64_t T = S_or_T;
    return dense_bwd_bytes(1, T, T, Hq, Hkv, D) + 2 * bounds_bytes(T) + order_bytes(T);
}

size_t sp_attn_varlen_fwd_workspace_bytes(int64_t T, int32_t Hq, int32_t Hkv, int32_t D,
                                          int32_t n_docs) {
    if (n_docs < 0) return 0;
    if (check_attn_shape(1, T, Hq, Hkv, D) != SP_OK || Hq == 0) return 0;
    const size_t n = 2 * bounds_bytes(T) + order_bytes(T);
    return n < 256 ? 256 : n;
}

sp_status sp_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B,
                      int64_t S, int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
                      void* hip_stream) {
    sp_status st = check_attn_shape(B, S, Hq, Hkv, D);
    if (st != SP_OK) return st;
    if (B == 0 || S == 0 || Hq == 0) return SP_OK;
    return run_dense_fwd(q, k, v, o, lse, B, S, S, 0, Hq, Hkv, D, sp::RowMap::attention_side(Hq, D),
                         sp::RowMap::attention_side(Hkv, D), softmax_scale, hip_stream);
}

sp_status sp_attn_fwd_seqlayout(const void* q, const void* k, const void* v, void* o, float* lse,
                                int64_t B, int64_t S_l, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                                float softmax_scale, void* hip_stream) {
    if (P <= 0 || S_l < 0) return SP_ERR_SHAPE;
    sp_status st = check_attn_shape(B, S_l * P, Hq, Hkv, D);
    if (st != SP_OK) return st;
    if (B == 0 || S_l == 0 || Hq == 0) return SP_OK;
    const int32_t lg = seq_chunk_log2(S_l);
    if (lg < 0) return SP_ERR_UNSUPPORTED;
    return run_dense_fwd(q, k, v, o, lse, B, S_l * P, S_l * P, 0, Hq, Hkv, D, sp::RowMap::sequence_side(lg, Hq, D, P),
                         sp::RowMap::sequence_side(lg, Hkv, D, P), softmax_scale, hip_stream);
}

sp_status sp_attn_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse,
                      const void* dO, void* dq, void* dk, void* dv, void* workspace,
                      size_t workspace_bytes, int64_t B, int64_t S, int32_t Hq, int32_t Hkv,
                      int32_t D, float softmax_scale, void* hip_stream) {
    return sp_attn_bwd_stages(q, k, v, o, lse, dO, dq, dk, dv, workspace, workspace_bytes, B, S, Hq,
                              Hkv, D, softmax_scale, SP_BWD_STAGE_ALL, hip_stream);
}

sp_status sp_attn_bwd_stages(const void* q, const void* k, const void* v, const void* o,
                             const float* lse, const void* dO, void* dq, void* dk, void* dv,
                             void* workspace, size_t workspace_bytes, int64_t B, int64_t S,
                             int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
                             int32_t stages, void* hip_stream) {
    sp_status st = check_attn_shape(B, S, Hq, Hkv, D);
    if (st != SP_OK) return st;
    if (stages <= 0 || (stages & ~SP_BWD_STAGE_ALL) != 0) return SP_ERR_SHAPE;
    if (B == 0 || S == 0 || Hq == 0) return SP_OK;
    const BwdBuffers t{q, k, v, o, lse, dO, dq, dk, dv, workspace, workspace_bytes};
    return run_dense_bwd(t, B, S, S, 0, Hq, Hkv, D, sp::RowMap::attention_side(Hq, D),
                         sp::RowMap::attention_side(Hkv, D), softmax_scale, stages, hip_stream);
}

sp_status sp_attn_bwd_seqlayout(const void* q, const void* k, const void* v, const void* o,
                                const float* lse, const void* dO, void* dq, void* dk, void* dv,
                                void* workspace, size_t workspace_bytes, int64_t B, int64_t S_l,
                                int32_t Hq, int32_t Hkv, int32_t D, int32_t P, float softmax_scale,
                                void* hip_stream) {
    if (P <= 0 || S_l < 0) return SP_ERR_SHAPE;
    const int64_t S = S_l * P;
    sp_status st = check_attn_shape(B, S, Hq, Hkv, D);
    if (st != SP_OK) return st;
    if (B == 0 || S == 0 || Hq == 0) return SP_OK;
    const int32_t lg = seq_chunk_log2(S_l);
    if (lg < 0) return SP_ERR_UNSUPPORTED;
    const BwdBuffers t{q, k, v, o, lse, dO, dq, dk, dv, workspace, workspace_bytes};
    return run_dense_bwd(t, B, S, S, 0, Hq, Hkv, D, sp::RowMap::sequence_side(lg, Hq, D, P),
                         sp::RowMap::sequence_side(lg, Hkv, D, P), softmax_scale, SP_BWD_STAGE_ALL, hip_stream);
}

namespace {
// common body of the two packed-document forward entry points; `workspace` holds at least
// sp_attn_varlen_fwd_workspace_bytes(...) bytes
sp_status run_varlen_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                         const int32_t* cu_seqlens, int32_t n_docs, int64_t T, int32_t Hq, int32_t Hkv, int32_t D,
                         float softmax_scale, void* workspace, hipStream_t s) {
    int32_t* row_lo = (int32_t*)workspace;
    int32_t* row_hi = (int32_t*)((char*)workspace + bounds_bytes(T));
    sp::AttnArgs a{};
    sp_status st = make_bounds(a, cu_seqlens, n_docs, T, row_lo, row_hi, (char*)row_hi + bounds_bytes(T), s);
    if (st != SP_OK) return st;
    a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
    a.B = 1; a.S = (int32_t)T; a.Hq = Hq; a.Hkv = Hkv; a.D = D;
    a.Skv = a.S; a.off = 0;
    attention_side_maps(a);
    a.scale = resolve_scale(softmax_scale, D);
    return sp::launch_attn_fwd(a, s);
}

// argument checks shared by the two entry points (everything but the workspace); SP_OK with *empty = true
// means "nothing to do"
sp_status check_varlen_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                           const int32_t* cu_seqlens, int32_t n_docs, int64_t T, int32_t Hq, int32_t Hkv, int32_t D,
                           bool* empty) {
    *empty = false;
    if (n_docs < 0) return SP_ERR_SHAPE;
    sp_status st = check_attn_shape(1, T, Hq, Hkv, D);
    if (st != SP_OK) return st;
    if (T == 0 || Hq == 0) { *empty = true; return SP_OK; }
    if (n_docs == 0) return SP_ERR_SHAPE;  // T > 0 rows must belong to some document
    if (!q || !k || !v || !o || !lse || !cu_seqlens) return SP_ERR_NULL;
    const void* ptrs[] = {q, k, v, o, lse};
    for (const void* p : ptrs)
        if (!sp::aligned16(p)) return SP_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(cu_seqlens) & 3u) != 0) return SP_ERR_ALIGN;
    return SP_OK;
}

// Scratch of sp_attn_varlen_fwd_static: device memory that belongs to the loaded library, one copy per
// device, held until the process ends.  In host code the array's name is only a handle; its device address
// is looked up once per device (with that device current) and kept.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};

sp_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SP_ERR_LAUNCH;
    if (dev < 0 || dev >= kMaxDevices) return SP_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return SP_ERR_LAUNCH;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SP_OK;
}
}  // namespace

sp_status sp_attn_varlen_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                             const int32_t* cu_seqlens, int32_t n_docs, int32_t max_seqlen,
                             int64_t T, int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    (void)max_seqlen;
    bool empty = false;
    sp_status st = check_varlen_fwd(q, k, v, o, lse, cu_seqlens, n_docs, T, Hq, Hkv, D, &empty);
    if (st != SP_OK || empty) return st;
    if (!workspace) return SP_ERR_NULL;
    if (!sp::aligned16(workspace)) return SP_ERR_ALIGN;
    if (workspace_bytes < sp_attn_varlen_fwd_workspace_bytes(T, Hq, Hkv, D, n_docs)) return SP_ERR_WORKSPACE;
    return run_varlen_fwd(q, k, v, o, lse, cu_seqlens, n_docs, T, Hq, Hkv, D, softmax_scale, workspace,
                          (hipStream_t)hip_stream);
}

sp_status sp_attn_varlen_fwd_static(const void* q, const void* k, const void* v, void* o, float* lse,
                                    const int32_t* cu_seqlens, int32_t n_docs, int32_t max_seqlen,
                                    int64_t T, int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
                                    void* hip_stream) {
    (void)max_seqlen;
    bool empty = false;
    sp_status st = check_varlen_fwd(q, k, v, o, lse, cu_seqlens, n_docs, T, Hq, Hkv, D, &empty);
    if (st != SP_OK || empty) return st;
    if (sp_attn_varlen_fwd_workspace_bytes(T, Hq, Hkv, D, n_docs) > kStaticScratchBytes) return SP_ERR_WORKSPACE;
    void* ws = nullptr;
    st = static_scratch(&ws);
    if (st != SP_OK) return st;
    // every word of the scratch that the attention kernel reads is written by the bounds kernels of this
    // call first, so nothing needs clearing between calls
    return run_varlen_fwd(q, k, v, o, lse, cu_seqlens, n_docs, T, Hq, Hkv, D, softmax_scale, ws,
                          (hipStream_t)hip_stream);
}

sp_status sp_varlen_check_cu_seqlens(const int32_t* cu_seqlens, int32_t n_docs, int64_t T, int32_t* flag,
                                     void* hip_stream) {
    if (n_docs < 0 || T < 0 || T >= (int64_t)1 << 31) return SP_ERR_SHAPE;
    if (!cu_seqlens || !flag) return SP_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(cu_seqlens) & 3u) != 0 || (reinterpret_cast<uintptr_t>(flag) & 3u) != 0)
        return SP_ERR_ALIGN;
    return sp::launch_check_cu_seqlens(cu_seqlens, n_docs, (int32_t)T, flag, (hipStream_t)hip_stream);
}

sp_status sp_attn_varlen_bwd(const void* q, const void* k, const void* v, const void* o,
                             const float* lse, const void* dO, void* dq, void* dk, void* dv,
                             const int32_t* cu_seqlens, int32_t n_docs, int32_t max_seqlen,
                             int64_t T, int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (n_docs < 0) return SP_ERR_SHAPE;
    sp_status st = check_attn_shape(1, T, Hq, Hkv, D);
    if (st != SP_OK) return st;
    if (T == 0 || Hq == 0) return SP_OK;
    if (n_docs == 0) return SP_ERR_SHAPE;
    if (!q || !k || !v || !o || !lse || !dO || !dq || !dk || !dv || !cu_seqlens || !workspace)
        return SP_ERR_NULL;
    const void* ptrs[] = {q, k, v, o, lse, dO, dq, dk, dv, workspace};
    for (const void* p : ptrs)
        if (!sp::aligned16(p)) return SP_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(cu_seqlens) & 3u) != 0) return SP_ERR_ALIGN;
    if (workspace_bytes < sp_attn_bwd_workspace_bytes(1, T, Hq, Hkv, D, n_docs)) return SP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    float* delta = (float*)workspace;
    float* aux = (float*)((char*)workspace + delta_bytes(T, Hq));
    int32_t* row_lo = (int32_t*)((char*)aux + 2 * aux_bytes(1, T, Hq));
    int32_t* row_hi = (int32_t*)((char*)row_lo + bounds_bytes(T));
    sp::AttnArgs a{};
    st = make_bounds(a, cu_seqlens, n_docs, T, row_lo, row_hi, (char*)row_hi + bounds_bytes(T), s);
    if (st != SP_OK) return st;
    a.q = q; a.k = k; a.v = v; a.o = const_cast<void*>(o); a.lse = const_cast<float*>(lse);
    a.dO = dO; a.dq = dq; a.dk = dk; a.dv = dv; a.delta = delta;
    a.aux = aux; a.S_pad = sp::aux_pitch(T);
    a.B = 1; a.S = (int32_t)T; a.Hq = Hq; a.Hkv = Hkv; a.D = D;
    a.Skv = a.S; a.off = 0;
    attention_side_maps(a);
    a.scale = resolve_scale(softmax_scale, D);
    a.stages = SP_BWD_STAGE_ALL;
    a.dkdv_splits = sp::dkdv_split_count(1, T, T, Hq, Hkv, max_seqlen);  // the hint only shapes the work split
    a.dkdv_part = a.dkdv_splits > 1 ? (float*)((char*)row_hi + bounds_bytes(T) + order_bytes(T)) : nullptr;
    return sp::launch_attn_bwd(a, s);
}

// ------------------------------------------------------------------ blockwise step of a ring schedule
namespace {
// 0 <= off, every key seen by some row; returns the offset clamped to "hides nothing"
sp_status check_block(int64_t B, int64_t Sq, int64_t Skv, int32_t Hq, int32_t Hkv, int32_t D, int64_t* off) {
    sp_status st = check_attn_shape(B, Sq, Hq, Hkv, D);
    if (st != SP_OK) return st;
    st = check_attn_shape(B, Skv, Hq, Hkv, D);
    if (st != SP_OK) return st;
    if (*off < 0) return SP_ERR_SHAPE;
    if (*off > Skv) *off = Skv;
    if (Sq > 0 && Skv > Sq + *off) return SP_ERR_SHAPE;
    return SP_OK;
}
}  // namespace

sp_status sp_attn_block_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B,
                            int64_t Sq, int64_t Skv, int32_t Hq, int32_t Hkv, int32_t D,
                            int64_t causal_offset, float softmax_scale, void* hip_stream) {
    sp_status st = check_block(B, Sq, Skv, Hq, Hkv, D, &causal_offset);
    if (st != SP_OK) return st;
    if (B == 0 || Sq == 0 || Hq == 0) return SP_OK;
    if (Skv == 0) return SP_ERR_SHAPE;  // rows that see no key have no softmax
    return run_dense_fwd(q, k, v, o, lse, B, Sq, Skv, causal_offset, Hq, Hkv, D, sp::RowMap::attention_side(Hq, D),
                         sp::RowMap::attention_side(Hkv, D), softmax_scale, hip_stream);
}

size_t sp_attn_block_bwd_workspace_bytes(int64_t B, int64_t Sq, int64_t Skv, int32_t Hq, int32_t Hkv, int32_t D) {
    if (B <= 0 || Sq <= 0 || Skv <= 0 || Hq <= 0) return 0;
    if (check_attn_shape(B, Sq, Hq, Hkv, D) != SP_OK || check_attn_shape(B, Skv, Hq, Hkv, D) != SP_OK) return 0;
    return dense_bwd_bytes(B, Sq, Skv, Hq, Hkv, D);
}

sp_status sp_attn_block_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse,
                            const void* dO, void* dq, void* dk, void* dv, void* workspace,
                            size_t workspace_bytes, int64_t B, int64_t Sq, int64_t Skv, int32_t Hq,
                            int32_t Hkv, int32_t D, int64_t causal_offset, float softmax_scale,
                            int32_t stages, void* hip_stream) {
    sp_status st = check_block(B, Sq, Skv, Hq, Hkv, D, &causal_offset);
    if (st != SP_OK) return st;
    if (stages <= 0 || (stages & ~SP_BWD_STAGE_ALL) != 0) return SP_ERR_SHAPE;
    if (B == 0 || Sq == 0 || Hq == 0) return SP_OK;
    if (Skv == 0) return SP_ERR_SHAPE;
    const BwdBuffers t{q, k, v, o, lse, dO, dq, dk, dv, workspace, workspace_bytes};
    return run_dense_bwd(t, B, Sq, Skv, causal_offset, Hq, Hkv, D, sp::RowMap::attention_side(Hq, D),
                         sp::RowMap::attention_side(Hkv, D), softmax_scale, stages, hip_stream);
}

sp_status sp_attn_merge(float* o_acc, float* lse_acc, const void* o_blk, const float* lse_blk, void* o_out,
                        int64_t B, int64_t S, int32_t Hq, int32_t D, void* hip_stream) {
    if (B < 0 || S < 0 || Hq < 0) return SP_ERR_SHAPE;
    if (D != 64 && D != 128) return SP_ERR_UNSUPPORTED;
    if (B * S >= (int64_t)1 << 31 || (Hq > 0 && B * S * Hq >= (int64_t)1 << 40)) return SP_ERR_SHAPE;
    if (B == 0 || S == 0 || Hq == 0) return SP_OK;
    if (!o_acc || !lse_acc || !o_blk || !lse_blk) return SP_ERR_NULL;
    if (!sp::aligned16(o_acc) || !sp::aligned16(lse_acc) || !sp::aligned16(o_blk) || !sp::aligned16(lse_blk) ||
        !sp::aligned16(o_out))
        return SP_ERR_ALIGN;
    return sp::launch_attn_merge(o_acc, lse_acc, o_blk, lse_blk, o_out, B, S, Hq, D, (hipStream_t)hip_stream);
}

// ------------------------------------------------------------------ pointwise operators outside attention
size_t sp_rmsnorm_bwd_workspace_bytes(int64_t T, int32_t C) {
    if (T <= 0 || C <= 0 || C % 8 != 0 || C > 8192) return 0;
    return align_up((size_t)sp::rmsnorm_bwd_groups(T) * (size_t)C * sizeof(float), 256);
}

sp_status sp_rmsnorm_fwd(const void* x, const void* w, void* y, float* rstd, int64_t T, int32_t C, float eps,
                         void* hip_stream) {
    if (T < 0 || C < 0 || !(eps >= 0.f)) return SP_ERR_SHAPE;
    if (C % 8 != 0 || C > 8192) return SP_ERR_UNSUPPORTED;
    if (T == 0 || C == 0) return SP_OK;
    if (!x || !w || !y || !rstd) return SP_ERR_NULL;
    if (!sp::aligned16(x) || !sp::aligned16(w) || !sp::aligned16(y) || !sp::aligned16(rstd)) return SP_ERR_ALIGN;
    if ((T + 3) / 4 > 0x7fffffff) return SP_ERR_SHAPE;
    return sp::launch_rmsnorm_fwd(x, w, y, rstd, T, C, eps, (hipStream_t)hip_stream);
}

sp_status sp_rmsnorm_bwd(const void* x, const void* w, const float* rstd, const void* dy, void* dx, void* dw,
                         void* workspace, size_t workspace_bytes, int64_t T, int32_t C, void* hip_stream) {
    if (T < 0 || C < 0) return SP_ERR_SHAPE;
    if (C % 8 != 0 || C > 8192) return SP_ERR_UNSUPPORTED;
    if (C == 0) return SP_OK;
    if (!x || !w || !rstd || !dy || !dx || !dw || !workspace) return SP_ERR_NULL;
    const void* ptrs[] = {x, w, rstd, dy, dx, dw, workspace};
    for (const void* p : ptrs)
        if (!sp::aligned16(p)) return SP_ERR_ALIGN;
    if (T == 0) return SP_ERR_SHAPE;  // dw of an empty batch is not defined by a launch-free call
    if (workspace_bytes < sp_rmsnorm_bwd_workspace_bytes(T, C)) return SP_ERR_WORKSPACE;
    return sp::launch_rmsnorm_bwd(x, w, rstd, dy, dx, dw, (float*)workspace, T, C, (hipStream_t)hip_stream);
}

sp_status sp_rope(const void* x, const float* cos_table, const float* sin_table, void* out, int64_t T, int32_t H,
                  int32_t D, int32_t conjugate, void* hip_stream) {
    if (T < 0 || H < 0 || D < 0) return SP_ERR_SHAPE;
    if (D % 16 != 0) return SP_ERR_UNSUPPORTED;
    if (T == 0 || H == 0 || D == 0) return SP_OK;
    if (!x || !cos_table || !sin_table || !out) return SP_ERR_NULL;
    if (!sp::aligned16(x) || !sp::aligned16(cos_table) || !sp::aligned16(sin_table) || !sp::aligned16(out))
        return SP_ERR_ALIGN;
    return sp::launch_rope(x, cos_table, sin_table, out, T, H, D, conjugate != 0, (hipStream_t)hip_stream);
}

sp_status sp_swiglu_fwd(const void* g, const void* u, void* y, int64_t n, void* hip_stream) {
    if (n < 0) return SP_ERR_SHAPE;
    if (n % 8 != 0) return SP_ERR_UNSUPPORTED;
    if (n == 0) return SP_OK;
    if (!g || !u || !y) return SP_ERR_NULL;
    if (!sp::aligned16(g) || !sp::aligned16(u) || !sp::aligned16(y)) return SP_ERR_ALIGN;
    return sp::launch_swiglu_fwd(g, u, y, n, (hipStream_t)hip_stream);
}

sp_status sp_swiglu_bwd(const void* g, const void* u, const void* dy, void* dg, void* du, int64_t n,
                        void* hip_stream) {
    if (n < 0) return SP_ERR_SHAPE;
    if (n % 8 != 0) return SP_ERR_UNSUPPORTED;
    if (n == 0) return SP_OK;
    if (!g || !u || !dy || !dg || !du) return SP_ERR_NULL;
    const void* ptrs[] = {g, u, dy, dg, du};
    for (const void* p : ptrs)
        if (!sp::aligned16(p)) return SP_ERR_ALIGN;
    return sp::launch_swiglu_bwd(g, u, dy, dg, du, n, (hipStream_t)hip_stream);
}

}  // extern "C"
