// Merge of two partial attention results over disjoint key sets (the update a
// device applies per arriving key/value block in a ring schedule, paper
// Section 4.1: keys and values are exchanged in p steps):
//   LSE = log(e^LSE_acc + e^LSE_blk)
//   O   = e^(LSE_acc - LSE) O_acc + e^(LSE_blk - LSE) O_blk
// The running result is kept in fp32 (O_acc, LSE_acc, updated in place) so that
// p merges round once; the block's O is the bf16 output of the forward kernel.
// Optionally the merged O is also written in bf16 (after the last block).
// HBM-bound: per element 4 + 2 bytes read, 4 (+ 2) written.
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;

template <int D>
__global__ __launch_bounds__(256) void attn_merge_kernel(float* __restrict__ o_acc, float* __restrict__ lse_acc,
                                                        const __bf16* __restrict__ o_blk,
                                                        const float* __restrict__ lse_blk, __bf16* __restrict__ o_out,
                                                        int64_t n_vec, int32_t S, int32_t Hq) {
    constexpr int LPV = D / 4;  // lanes per (row, head) vector, 4 elements each: a wave's fp32 loads and stores
                                // are 1 KB contiguous (8 elements per lane would stride them by 32 bytes)
    const int64_t vec = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPV;  // (b*S + i)*Hq + h
    const int part = threadIdx.x % LPV;
    if (vec >= n_vec) return;
    const int64_t bi = vec / Hq, b = bi / S;
    const int32_t h = (int32_t)(vec - bi * Hq), i = (int32_t)(bi - b * S);
    const int64_t li = (b * Hq + h) * S + i;
    const float la = lse_acc[li], lb = lse_blk[li];
    const float m = fmaxf(la, lb);
    float wa = 0.f, wb = 0.f, l = -INFINITY;
    if (m > -INFINITY) {  // some key has been seen
        const float ea = expf(la - m), eb = expf(lb - m);
        const float inv = 1.0f / (ea + eb);
        wa = ea * inv; wb = eb * inv;
        l = m + logf(ea + eb);
    }
    const size_t at = (size_t)vec * D + 4 * part;
    // plain accesses on purpose: O_acc is updated in place, and non-temporal loads and stores of the same
    // lines measured 6 % slower
    const f32x4 a0 = *reinterpret_cast<const f32x4*>(o_acc + at);
    const bf16x4 bb = __builtin_bit_cast(bf16x4, *reinterpret_cast<const u32x2*>(o_blk + at));
    f32x4 r0;
#pragma unroll
    for (int e = 0; e < 4; ++e) r0[e] = wa * a0[e] + wb * (float)bb[e];
    *reinterpret_cast<f32x4*>(o_acc + at) = r0;
    if (o_out) {
        u32x2 w;
        w[0] = pack_bf16(r0[0], r0[1]); w[1] = pack_bf16(r0[2], r0[3]);
        *reinterpret_cast<u32x2*>(o_out + at) = w;
    }
    // every lane of the vector has read LSE_acc above (the lanes of a vector sit in one wave)
    if (part == 0) lse_acc[li] = l;
}

}  // namespace

namespace sp {

sp_status launch_attn_merge(float* o_acc, float* lse_acc, const void* o_blk, const float* lse_blk, void* o_out,
                            int64_t B, int64_t S, int32_t Hq, int32_t D, hipStream_t st) {
    const int64_t n_vec = B * S * Hq;
    const int64_t blocks = (n_vec * (D / 4) + 255) / 256;
    if (blocks > 0x7fffffff) return SP_ERR_SHAPE;
    if (D == 128)
        hipLaunchKernelGGL((attn_merge_kernel<128>), dim3((unsigned)blocks), dim3(256), 0, st, o_acc, lse_acc,
                           (const __bf16*)o_blk, lse_blk, (__bf16*)o_out, n_vec, (int32_t)S, Hq);
    else if (D == 64)
        hipLaunchKernelGGL((attn_merge_kernel<64>), dim3((unsigned)blocks), dim3(256), 0, st, o_acc, lse_acc,
                           (const __bf16*)o_blk, lse_blk, (__bf16*)o_out, n_vec, (int32_t)S, Hq);
    else
        return SP_ERR_UNSUPPORTED;
    return launch_status();
}

}  // namespace sp
