/*
 * sp_hotpath.h -- C ABI of the per-GPU hot path of a Ulysses-style
 * sequence-parallel transformer layer on one MI355X (gfx950).
 *
 * The paper (Section 2, Figure 1) describes the step this library serves:
 * outside attention a device holds part of the sequence with all heads,
 * [S/P, H, D]; an all-to-all re-shards to the whole sequence with a subset of
 * the heads, [S, H/P, D]; attention runs locally on those heads; a second
 * all-to-all restores the first layout.  This library is what one device
 * executes around and between those two exchanges: the local re-layout that
 * makes the P per-peer messages contiguous (and its inverse), and causal
 * grouped-query attention, forward and backward, over the full sequence for
 * the device's head shard.  The exchange itself is not part of it.
 *
 * Conventions, all entry points
 *   - Every pointer is a DEVICE pointer unless stated otherwise, 16-byte
 *     aligned; tensors are dense row-major with the head dim innermost.
 *   - The caller owns every buffer.  The library allocates nothing, frees
 *     nothing and never synchronises: a call validates its arguments on the
 *     host, enqueues kernels on `hip_stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and returns.
 *   - Outputs are fully overwritten; they need no pre-clearing.
 *   - Inputs and outputs must not overlap.
 *   - Errors are return codes.  Argument errors are found before any launch
 *     (no GPU is needed to get them); a failed launch gives SP_ERR_LAUNCH.
 *   - Empty problems (a zero extent) return SP_OK without launching.
 *   - No global mutable state (sp_attn_varlen_fwd_static excepted, see there):
 *     calls from several host threads are safe as long as they do not share
 *     output or workspace buffers.
 *   - bf16 tensors are `uint16_t`-sized elements passed as `const void*`.
 */
#ifndef SP_HOTPATH_H
#define SP_HOTPATH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SP_OK = 0,
    SP_ERR_NULL = 1,        /* a required pointer is NULL                        */
    SP_ERR_SHAPE = 2,       /* negative extent, H % P != 0, Hq % Hkv != 0, ...   */
    SP_ERR_UNSUPPORTED = 3, /* head dim or element size outside the supported set */
    SP_ERR_WORKSPACE = 4,   /* workspace smaller than the matching *_bytes query  */
    SP_ERR_ALIGN = 5,       /* a pointer is not 16-byte aligned                   */
    SP_ERR_LAUNCH = 6       /* the HIP runtime refused a launch                   */
} sp_status;

/* Static, human-readable name of a status code.  Never NULL. */
const char* sp_status_str(sp_status s);

/* Version of this ABI (bumped on any signature change and when a workspace requirement grows). */
int32_t sp_abi_version(void);

/* ---------------------------------------------------------------------------
 * Re-layout before the first all-to-all (Section 2: the exchange re-shards
 * from the sequence dimension to the head dimension; Section 3.1, challenge 1:
 * the exchange needs token buffers of a size fixed by batch, sequence length
 * and model dimension).
 *
 *   in  [B, S_l, H, D]      this device's S_l = S/P tokens, all H heads
 *   out [B, P*S_l, H/P, D]  out[b, p*S_l + s, j, :] = in[b, s, p*(H/P) + j, :]
 *
 * Rows p*S_l .. (p+1)*S_l-1 of `out` are the contiguous message for peer p
 * (heads are split into P contiguous groups, so a query-head group and its
 * key/value head land on the same peer when both head counts divide by P).
 * Seen from the receiving side, the P messages a device gets, concatenated in
 * source-rank order, are its [S, H/P, D] attention-side tensor.
 *
 * A pure byte permutation, bit-exact for any element contents.
 * elem_bytes in {2, 4}; D*elem_bytes must be a multiple of 16; H % P == 0.
 * ------------------------------------------------------------------------- */
sp_status sp_pack_seq_to_head(const void* in, void* out, int64_t B, int64_t S_l, int64_t H,
                              int64_t D, int32_t P, int32_t elem_bytes, void* hip_stream);

/* Exact inverse, applied after the second all-to-all (Section 2: tokens go
 * "back to their original input sizes"); it is also the gradient of the pack
 * (Section 3.1: every inserted node needs its conjugate gradient operator).
 *
 *   in  [B, P*S_l, H/P, D]
 *   out [B, S_l, H, D]      out[b, s, p*(H/P) + j, :] = in[b, p*S_l + s, j, :]
 */
sp_status sp_unpack_head_to_seq(const void* in, void* out, int64_t B, int64_t S_l, int64_t H,
                                int64_t D, int32_t P, int32_t elem_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------
 * Causal grouped-query attention, forward (Section 2: each device computes
 * attention locally on its heads over the entire context; Section 3.1,
 * challenge 3: the causal mask is part of the model; Section 4: evaluated
 * models use grouped-query or full attention).
 *
 *   q [B, S, Hq, D], k, v [B, S, Hkv, D]   bf16
 *   o [B, S, Hq, D]                        bf16 (round-to-nearest-even)
 *   lse [B, Hq, S]                         fp32, natural log, scale included
 *
 * Query head a reads key/value head a / (Hq/Hkv).  Key j is visible to query
 * i iff j <= i.  s_ij = softmax_scale * q_i.k_j; softmax_scale <= 0 selects
 * 1/sqrt(D).  Contractions run in bf16 MFMA with fp32 accumulation; the
 * softmax runs in fp32.  D in {64, 128}; Hq % Hkv == 0; S < 2^31.
 * ------------------------------------------------------------------------- */
sp_status sp_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                      int64_t B, int64_t S, int32_t Hq, int32_t Hkv, int32_t D,
                      float softmax_scale, void* hip_stream);

/* Bytes of device workspace sp_attn_bwd / sp_attn_varlen_fwd / sp_attn_varlen_bwd
 * need for these extents.  Dense call: pass B and S, n_docs = 0.  Packed
 * documents: pass the total row count T as S_or_T and n_docs > 0; B is ignored
 * then (pass 1).  Returns 0 for invalid arguments, B <= 0 included. */
size_t sp_attn_bwd_workspace_bytes(int64_t B, int64_t S_or_T, int32_t Hq, int32_t Hkv, int32_t D,
                                   int32_t n_docs);
size_t sp_attn_varlen_fwd_workspace_bytes(int64_t T, int32_t Hq, int32_t Hkv, int32_t D,
                                          int32_t n_docs);

/* ---------------------------------------------------------------------------
 * Backward of sp_attn_fwd (Section 3.1: the rewritten graph must stay correct
 * in the backward pass; Section 4.2 (breakdown analysis): the backward is where recomputation
 * under activation checkpointing is paid).
 *
 *   inputs : q, k, v, o (as written by the forward), lse, dO [B, S, Hq, D] bf16
 *   outputs: dq [B, S, Hq, D], dk, dv [B, S, Hkv, D]  bf16
 *   workspace: >= sp_attn_bwd_workspace_bytes(...) bytes, contents undefined
 *              on entry and exit (holds Delta_i = dO_i.O_i in fp32, per-row
 *              accumulator seeds, and fp32 partial sums of dK/dV when a key
 *              tile's work is shared by several workgroups).
 *
 *   dV_j = sum_{a in group} sum_{i>=j} P_ij dO_i,  dP_ij = dO_i.v_j,
 *   dS_ij = P_ij (dP_ij - Delta_i),
 *   dQ_i = scale sum_{j<=i} dS_ij k_j,  dK_j = scale sum_{a in group} sum_{i>=j} dS_ij q_i.
 *
 * No atomics: results are bitwise reproducible run to run.
 * ------------------------------------------------------------------------- */
sp_status sp_attn_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse,
                      const void* dO, void* dq, void* dk, void* dv, void* workspace,
                      size_t workspace_bytes, int64_t B, int64_t S, int32_t Hq, int32_t Hkv,
                      int32_t D, float softmax_scale, void* hip_stream);

/* The same backward, one stage at a time.  `stages` is a bit mask of
 * SP_BWD_STAGE_*; the stages of one backward must run in the order delta, then
 * dkdv and dq (those two are independent of each other), all with the same
 * arguments and workspace.  sp_attn_bwd(...) == stages SP_BWD_STAGE_ALL.
 * Meant for per-stage timing and for callers that schedule the stages
 * themselves. */
enum { SP_BWD_STAGE_DELTA = 1, SP_BWD_STAGE_DKDV = 2, SP_BWD_STAGE_DQ = 4, SP_BWD_STAGE_ALL = 7 };
sp_status sp_attn_bwd_stages(const void* q, const void* k, const void* v, const void* o,
                             const float* lse, const void* dO, void* dq, void* dk, void* dv,
                             void* workspace, size_t workspace_bytes, int64_t B, int64_t S,
                             int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
                             int32_t stages, void* hip_stream);

/* ---------------------------------------------------------------------------
 * The same attention, forward and backward, on SEQUENCE-SIDE tensors: the pack
 * of Q, K, V (and dO) and the unpack of O (and dQ, dK, dV) folded into the
 * attention kernels' own loads and stores, so that no re-laid-out copy is ever
 * written to memory (Section 2, Figure 1: the two layouts on either side of
 * the exchange; on one device, what the exchange would move is read in place).
 *
 *   q, o, dO, dq [B, S_l, P*Hq, D]; k, v, dk, dv [B, S_l, P*Hkv, D]   bf16
 *   lse [B, Hq, P*S_l]                                                 fp32
 *
 * Hq, Hkv are the per-peer head counts.  The result is, bit for bit,
 *   unpack(sp_attn_fwd(pack(q), pack(k), pack(v)))  resp. the unpacked
 * gradients of sp_attn_bwd on the packed tensors: attention row p*S_l + s,
 * head j is sequence-side row s, head p*H + j.
 * S_l must be a power of two >= 256 (no tile of any kernel may straddle two
 * peers' chunks): SP_ERR_UNSUPPORTED otherwise.  Workspace of the backward:
 * sp_attn_bwd_workspace_bytes(B, P*S_l, Hq, Hkv, D, 0).
 * ------------------------------------------------------------------------- */
sp_status sp_attn_fwd_seqlayout(const void* q, const void* k, const void* v, void* o, float* lse,
                                int64_t B, int64_t S_l, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                                float softmax_scale, void* hip_stream);
sp_status sp_attn_bwd_seqlayout(const void* q, const void* k, const void* v, const void* o,
                                const float* lse, const void* dO, void* dq, void* dk, void* dv,
                                void* workspace, size_t workspace_bytes, int64_t B, int64_t S_l,
                                int32_t Hq, int32_t Hkv, int32_t D, int32_t P, float softmax_scale,
                                void* hip_stream);

/* ---------------------------------------------------------------------------
 * One step of a ring schedule (the second sequence-parallel scheme the paper
 * measures, Section 4 baselines and Section 4.1: the sequence stays sharded and
 * key/value blocks are passed from device to device in p steps).  Per arriving
 * block a device computes the attention of its query block against that block
 * and merges it into a running result; in the backward pass it computes the
 * block pair's share of the gradients.
 *
 *   q, o, dO, dq [B, Sq, Hq, D]; k, v, dk, dv [B, Skv, Hkv, D]   bf16
 *   lse [B, Hq, Sq]                                               fp32
 *
 * Query row i sees keys j <= i + causal_offset.  With the query block starting
 * at global position a and the key block at global position c, causal
 * attention over the whole sequence is causal_offset = a - c: 0 for the
 * diagonal block, anything >= Skv - 1 hides nothing (a block from the past);
 * blocks from the future are not computed at all.  Required: causal_offset >= 0
 * and Skv <= Sq + causal_offset (every key is seen by some row); SP_ERR_SHAPE
 * otherwise.  sp_attn_fwd is the case Skv = Sq, causal_offset = 0, bit for bit.
 *
 * sp_attn_block_fwd: o, lse of the block alone (the softmax runs over the
 *   visible keys of this block only).
 * sp_attn_merge: folds a block's (o_blk bf16, lse_blk) into the running
 *   (o_acc fp32 [B, S, Hq, D], lse_acc fp32 [B, Hq, S]), in place:
 *     lse = log(e^lse_acc + e^lse_blk),
 *     o   = e^(lse_acc - lse) o_acc + e^(lse_blk - lse) o_blk.
 *   The caller starts from o_acc = 0, lse_acc = -inf.  If o_out is not NULL the
 *   merged O is also written there in bf16 (pass it with the last block).
 * sp_attn_block_bwd: dq, dk, dv = this block pair's shares (bf16; the caller
 *   adds the dq shares over key blocks and the dk, dv shares over query
 *   blocks).  o and lse are the FINAL (merged) ones of the query rows, dO the
 *   gradient of the final O.  `stages` as in sp_attn_bwd_stages: the delta
 *   stage depends on o, dO, lse only, so a caller looping over key blocks may
 *   run it once (SP_BWD_STAGE_ALL on the first block) and pass
 *   SP_BWD_STAGE_DKDV | SP_BWD_STAGE_DQ with the same workspace afterwards.
 *   Workspace: sp_attn_block_bwd_workspace_bytes (0 for invalid extents).
 * Outputs are fully overwritten; nothing is allocated; same error behaviour as
 * the entry points above.
 * ------------------------------------------------------------------------- */
sp_status sp_attn_block_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t B,
                            int64_t Sq, int64_t Skv, int32_t Hq, int32_t Hkv, int32_t D,
                            int64_t causal_offset, float softmax_scale, void* hip_stream);
sp_status sp_attn_merge(float* o_acc, float* lse_acc, const void* o_blk, const float* lse_blk, void* o_out,
                        int64_t B, int64_t S, int32_t Hq, int32_t D, void* hip_stream);
size_t sp_attn_block_bwd_workspace_bytes(int64_t B, int64_t Sq, int64_t Skv, int32_t Hq, int32_t Hkv,
                                         int32_t D);
sp_status sp_attn_block_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse,
                            const void* dO, void* dq, void* dk, void* dv, void* workspace,
                            size_t workspace_bytes, int64_t B, int64_t Sq, int64_t Skv, int32_t Hq,
                            int32_t Hkv, int32_t D, int64_t causal_offset, float softmax_scale,
                            int32_t stages, void* hip_stream);

/* ---------------------------------------------------------------------------
 * Packed variable-length documents (not in the paper; the block-diagonal form
 * of the same operator, as long-context training batches are usually packed).
 *
 *   q [T, Hq, D], k, v [T, Hkv, D], o [T, Hq, D] bf16; lse [Hq, T] fp32
 *   cu_seqlens: DEVICE int32 [n_docs+1], cu[0] = 0, non-decreasing,
 *               cu[n_docs] = T.  Rows [cu[t], cu[t+1]) are document t; key j is
 *               visible to query i iff both are in one document and j <= i.
 *               Empty documents are allowed.  The contents are read on the
 *               device only; a malformed array is undefined behaviour confined
 *               to the output values (all accesses stay inside [0, T)).
 *   max_seqlen: host upper bound on the longest document (a hint; 0 = T).  It
 *               never changes a result beyond rounding order: the backward uses
 *               it to decide over how many workgroups a key tile's work is
 *               spread (short documents want fewer).
 *   workspace : >= the matching *_workspace_bytes query.  It receives the
 *               per-row document windows and the order in which workgroups
 *               take the 256-row tiles (longest first: with documents of
 *               mixed lengths a tile's work does not follow from its position).
 * ------------------------------------------------------------------------- */
sp_status sp_attn_varlen_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                             const int32_t* cu_seqlens, int32_t n_docs, int32_t max_seqlen,
                             int64_t T, int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

sp_status sp_attn_varlen_bwd(const void* q, const void* k, const void* v, const void* o,
                             const float* lse, const void* dO, void* dq, void* dk, void* dv,
                             const int32_t* cu_seqlens, int32_t n_docs, int32_t max_seqlen,
                             int64_t T, int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/* Debug aid for the packed-document calls, which read cu_seqlens on the device only and so cannot reject a
 * malformed array on the host: one small kernel writes to *flag (DEVICE int32, 4-byte aligned) 0 when
 * cu_seqlens (n_docs + 1 entries) starts at 0, never decreases and ends at T, else a bit mask:
 * 1 = cu[0] != 0, 2 = some cu[t+1] < cu[t], 4 = cu[n_docs] != T.  Nothing else depends on it; the caller
 * reads the flag back when it wants to (the call itself does not synchronise). */
sp_status sp_varlen_check_cu_seqlens(const int32_t* cu_seqlens, int32_t n_docs, int64_t T, int32_t* flag,
                                     void* hip_stream);

/* sp_attn_varlen_fwd for callers that cannot allocate device memory at all, not
 * even a workspace: code recorded into a HIP graph, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments minus the workspace, same kernels, same
 * bits.  The document windows and tile orders go to a scratch array of 8 MiB
 * (8,388,608 bytes) that is part of the loaded library: every device the library
 * runs on holds one copy until the process ends.  A problem whose
 * sp_attn_varlen_fwd_workspace_bytes(...) exceeds that size (about one million
 * rows) gets SP_ERR_WORKSPACE and launches nothing.  The first call on a device
 * looks up that device's copy (no allocation); SP_ERR_UNSUPPORTED for a device
 * ordinal above 63.  All calls on one device share the one array: calls that
 * may overlap in time on one device (two streams, two host threads) race on it
 * and must be serialised by the caller; calls ordered on one stream are safe,
 * each call rewrites every word it later reads. */
sp_status sp_attn_varlen_fwd_static(const void* q, const void* k, const void* v, void* o, float* lse,
                                    const int32_t* cu_seqlens, int32_t n_docs, int32_t max_seqlen,
                                    int64_t T, int32_t Hq, int32_t Hkv, int32_t D, float softmax_scale,
                                    void* hip_stream);

/* ---------------------------------------------------------------------------
 * Pointwise operators between the matrix multiplications of a Llama layer, on
 * one device's token shard [T = S/P tokens, full model dimension] (Section 2,
 * Figure 1: outside attention a device holds part of the sequence with all of
 * the model dimension).  The paper's activation-checkpointing strategy lets
 * every operator outside the attention layer be rematerialised in the backward
 * pass (Section 3.2), so each forward below runs twice per training step; the
 * evaluated models are Llama models (Section 4 setup), whose published layer
 * these operators come from.  bf16 in and out, fp32 arithmetic, one rounding.
 *
 * RMS norm:  y[t,c] = x[t,c] * rstd[t] * w[c],  rstd[t] = 1/sqrt(mean_c x[t,c]^2 + eps)
 *   forward : x, y [T, C] bf16, w [C] bf16, rstd [T] fp32 (output, kept for the backward)
 *   backward: dx = g*rstd - x*rstd^3*(sum_c g x)/C with g = dy*w;  dw = sum_t dy*x*rstd
 *             dx [T, C], dw [C] bf16 (fp32 accumulation, fixed summation order);
 *             workspace >= sp_rmsnorm_bwd_workspace_bytes(T, C), contents undefined.
 *   C % 8 == 0 and C <= 8192 (SP_ERR_UNSUPPORTED otherwise).
 *
 * Rotary embedding:  x, out [T, H, D] bf16; cos_table, sin_table [T, D/2] fp32 hold
 *   the cosine and sine of the angle of (token t, pair i).  Element i of the first
 *   half of the head dim and element i of the second half form a pair:
 *     out1 = x1*cos - x2*sin,  out2 = x2*cos + x1*sin.
 *   conjugate != 0 rotates by the negative angle: the gradient operator.  out may
 *   be x itself (in place); any other overlap is not allowed.  D % 16 == 0.
 *
 * SwiGLU gate:  y = g*sigmoid(g)*u over n = T*F elements (n % 8 == 0);
 *   backward: dg = dy*u*s*(1 + g*(1 - s)), du = dy*g*s with s = sigmoid(g).
 * ------------------------------------------------------------------------- */
size_t sp_rmsnorm_bwd_workspace_bytes(int64_t T, int32_t C);
sp_status sp_rmsnorm_fwd(const void* x, const void* w, void* y, float* rstd, int64_t T, int32_t C, float eps,
                         void* hip_stream);
sp_status sp_rmsnorm_bwd(const void* x, const void* w, const float* rstd, const void* dy, void* dx, void* dw,
                         void* workspace, size_t workspace_bytes, int64_t T, int32_t C, void* hip_stream);
sp_status sp_rope(const void* x, const float* cos_table, const float* sin_table, void* out, int64_t T, int32_t H,
                  int32_t D, int32_t conjugate, void* hip_stream);
sp_status sp_swiglu_fwd(const void* g, const void* u, void* y, int64_t n, void* hip_stream);
sp_status sp_swiglu_bwd(const void* g, const void* u, const void* dy, void* dg, void* du, int64_t n,
                        void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SP_HOTPATH_H */
