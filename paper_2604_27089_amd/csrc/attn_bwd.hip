// Causal grouped-query attention, backward, for one device's head shard
// (paper Section 3.1: the rewritten graph must stay correct in the backward
// pass, each inserted operator having a gradient; Section 4.2 (breakdown analysis): under
// activation checkpointing the backward is where the extra time goes).
//
// Three stages, no atomics (bitwise reproducible):
//   delta : Delta_i = dO_i . O_i and the per-row seeds -LSE_i/scale, -Delta_i
//           (this file; HBM-bound, fp32 out)
//   dkdv  : attn_bwd_dkdv.hip
//   dq    : attn_bwd_dq.hip
// P is rebuilt from the saved LSE: P_ij = exp(scale*s_ij - LSE_i); S and dP
// are evaluated in both matrix kernels.
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;


// ------------------------------------------------------------------ delta
// One 16-byte vector of O and dO per lane, D/8 lanes per (row, head).  The grid covers the padded row range
// [0, S_pad): rows past the sequence only zero their slots of the per-row scalars (they are fetched by the
// dK/dV kernel, never used unmasked).
template <int D>
__global__ __launch_bounds__(256) void delta_kernel(const __bf16* __restrict__ o,
                                                   const __bf16* __restrict__ dO,
                                                   const float* __restrict__ lse,
                                                   float* __restrict__ delta, float* __restrict__ aux,
                                                   int32_t B, int32_t S, int32_t S_pad, int32_t Hq,
                                                   float inv_scale, RowMap map) {
    constexpr int LPV = D / 8;  // lanes per (row, head) vector, 16 bytes each
    const int64_t n_vec = (int64_t)B * S_pad * Hq;
    const int64_t vec = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPV;  // (b*S_pad + i)*Hq + h
    const int part = threadIdx.x % LPV;
    if (vec >= n_vec) return;  // whole (row, head) groups of lanes leave together: LPV divides 64
    const int64_t bi = vec / Hq, b = bi / S_pad;
    const int32_t h = (int32_t)(vec - bi * Hq), i = (int32_t)(bi - b * S_pad);
    // the per-row accumulator seeds of the dK/dV kernel: per 32-row tile, 32 x -LSE/scale then 32 x -Delta
    float* t = aux + ((b * Hq + h) * (S_pad / 32) + i / 32) * 64 + i % 32;
    if (i >= S) {
        if (part == 0) { t[0] = 0.f; t[32] = 0.f; }
        return;
    }
    const size_t at = (size_t)b * S * Hq * D + map.off(i) + (size_t)h * D + 8 * part;
    const bf16x8 x = as_bf16x8(*reinterpret_cast<const u32x4*>(o + at));
    const bf16x8 y = as_bf16x8(*reinterpret_cast<const u32x4*>(dO + at));
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)x[e] * (float)y[e];
#pragma unroll
    for (int off = LPV / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (part == 0) {
        delta[(b * Hq + h) * S + i] = acc;
        t[0] = -lse[(b * Hq + h) * S + i] * inv_scale;
        t[32] = -acc;
    }
}

template <int D, bool VARLEN>
sp_status launch(const AttnArgs& a, hipStream_t st) {
    if (a.stages & SP_BWD_STAGE_DELTA) {
        const int64_t lanes = (int64_t)a.B * a.S_pad * a.Hq * (D / 8);
        const int64_t blocks = (lanes + 255) / 256;
        if (blocks > 0x7fffffff) return SP_ERR_SHAPE;
        hipLaunchKernelGGL((delta_kernel<D>), dim3((unsigned)blocks), dim3(256), 0, st, (const __bf16*)a.o,
                           (const __bf16*)a.dO, a.lse, a.delta, a.aux, a.B, a.S, a.S_pad, a.Hq,
                           1.0f / a.scale, a.qmap);
        if (hipGetLastError() != hipSuccess) return SP_ERR_LAUNCH;
    }
    if (a.stages & SP_BWD_STAGE_DKDV) {
        const sp_status r = launch_attn_bwd_dkdv(a, st);
        if (r != SP_OK) return r;
    }
    if (a.stages & SP_BWD_STAGE_DQ) {
        const sp_status r = launch_attn_bwd_dq(a, st);
        if (r != SP_OK) return r;
    }
    return SP_OK;
}

}  // namespace

namespace sp {

sp_status launch_attn_bwd(const AttnArgs& a, hipStream_t st) {
    if (a.Hq > 65535 || a.B > 65535) return SP_ERR_SHAPE;
    const bool varlen = a.row_lo != nullptr;
    if (a.D == 128) return varlen ? launch<128, true>(a, st) : launch<128, false>(a, st);
    if (a.D == 64) return varlen ? launch<64, true>(a, st) : launch<64, false>(a, st);
    return SP_ERR_UNSUPPORTED;
}

}  // namespace sp
