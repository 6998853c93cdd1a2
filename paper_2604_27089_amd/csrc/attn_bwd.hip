// Causal grouped-query attention, backward, for one device's head shard
// (paper Section 3.1: the rewritten graph must stay correct in the backward
// pass, each inserted operator having a gradient; Section 4.4: under
// activation checkpointing the backward is where the extra time goes).
//
// Three kernels, no atomics (bitwise reproducible):
//   delta : Delta_i = dO_i . O_i                     (HBM-bound, fp32 out)
//   dkdv  : one workgroup per 128 keys of one KV head; each wave keeps K and V
//           of its 32 keys resident as MFMA B operands and dK, dV as
//           accumulators; it streams Q/dO tiles of the G query heads of the
//           group through LDS (row-major for S = Q.K^T and dP = dO.V^T, and
//           transposed for dV += P^T.dO and dK += dS^T.Q).
//   dq    : one workgroup per 128 query rows of one query head (same shape as
//           the forward): Q and dO resident, K/V tiles through LDS,
//           dQ^T += K^T . dS^T.
// P is rebuilt from the saved LSE: P_ij = exp(scale*s_ij - LSE_i); S and dP
// are evaluated in both kernels.
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;

constexpr int kThreads = 256;

// ------------------------------------------------------------------ delta
template <int D>
__global__ __launch_bounds__(256) void delta_kernel(const __bf16* __restrict__ o,
                                                   const __bf16* __restrict__ dO,
                                                   const float* __restrict__ lse,
                                                   float* __restrict__ delta, float* __restrict__ lsn,
                                                   float* __restrict__ dn, int32_t B, int32_t S,
                                                   int32_t S_pad, int32_t Hq, float inv_scale) {
    constexpr int LPV = D / 8;  // lanes per (row, head) vector, 16 bytes each
    const int64_t n_vec = (int64_t)B * S * Hq;
    const int64_t vec = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPV;
    const int part = threadIdx.x % LPV;
    float acc = 0.f;
    if (vec < n_vec) {
        const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(o + vec * D + 8 * part));
        const bf16x8 b = as_bf16x8(*reinterpret_cast<const u32x4*>(dO + vec * D + 8 * part));
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
    }
#pragma unroll
    for (int off = LPV / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (vec < n_vec && part == 0) {
        const int64_t bi = vec / Hq;  // b*S + i
        const int32_t h = (int32_t)(vec - bi * Hq);
        const int64_t b = bi / S;
        const int32_t i = (int32_t)(bi - b * S);
        delta[(b * Hq + h) * S + i] = acc;
        // the per-row accumulator seeds of the dK/dV kernel
        lsn[(b * Hq + h) * S_pad + i] = -lse[(b * Hq + h) * S + i] * inv_scale;
        dn[(b * Hq + h) * S_pad + i] = -acc;
    }
}

// zero the padding rows [S, S_pad) of the per-row scalars (they are fetched, never used unmasked)
__global__ __launch_bounds__(256) void aux_pad_kernel(float* __restrict__ lsn, float* __restrict__ dn,
                                                     int32_t BH, int32_t S, int32_t S_pad) {
    const int32_t pad = S_pad - S;
    const int64_t n = (int64_t)BH * pad;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n) return;
    const int64_t bh = t / pad;
    const int32_t i = S + (int32_t)(t - bh * pad);
    lsn[bh * S_pad + i] = 0.f;
    dn[bh * S_pad + i] = 0.f;
}

struct BwdParams {
    const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* dO;
    const float* lse; const float* delta;
    __bf16* dq; __bf16* dk; __bf16* dv;
    const int32_t* row_lo; const int32_t* row_hi;
    int32_t S, Hq, Hkv, G, n_tiles;
    float scale, scale_log2;
};

// ------------------------------------------------------------------ dQ
constexpr int DQ_BM = 128;  // query rows per workgroup (32 per wave)
constexpr int DQ_BN = 64;   // keys per tile

template <int D>
struct DqSmem {
    static constexpr int LDR = D + 8;
    static constexpr int LDT = DQ_BN + 8;
    __bf16 k[DQ_BN * LDR];
    __bf16 v[DQ_BN * LDR];
    __bf16 kt[D * LDT];
};

template <int D, bool VARLEN>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_kernel(BwdParams p) {
    constexpr int KCH = D / 8;
    constexpr int V_LOADS = DQ_BN * KCH / kThreads;
    constexpr int TASKS = (DQ_BN / 4) * KCH;
    constexpr int LDR = DqSmem<D>::LDR, LDT = DqSmem<D>::LDT;
    __shared__ DqSmem<D> sm;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
    const int qt = p.n_tiles - 1 - (int)blockIdx.x;
    const int h = blockIdx.y, b = blockIdx.z, g = h / p.G;
    const int S = p.S;
    const size_t q_row_stride = (size_t)p.Hq * D, kv_row_stride = (size_t)p.Hkv * D;
    const __bf16* qb = p.q + ((size_t)b * S * p.Hq + h) * D;
    const __bf16* dob = p.dO + ((size_t)b * S * p.Hq + h) * D;
    const __bf16* kb = p.k + ((size_t)b * S * p.Hkv + g) * D;
    const __bf16* vb = p.v + ((size_t)b * S * p.Hkv + g) * D;

    const int i0 = qt * DQ_BM;
    const int wrow0 = i0 + 32 * wave;
    const int qrow = wrow0 + lo;
    const int qrow_c = qrow < S ? qrow : S - 1;

    bf16x8 qreg[D / 16], doreg[D / 16];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
        qreg[kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(qb + (size_t)qrow_c * q_row_stride + 16 * kk + 8 * hi));
        doreg[kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(dob + (size_t)qrow_c * q_row_stride + 16 * kk + 8 * hi));
    }
    const float lse2 = p.lse[((size_t)b * p.Hq + h) * S + qrow_c] * kLog2e;
    const float delta = p.delta[((size_t)b * p.Hq + h) * S + qrow_c];

    int row_lo = 0, wave_lo_min = 0, wave_lo_max = 0, wg_lo_min = 0;
    if (VARLEN) {
        row_lo = p.row_lo[qrow_c];
        wave_lo_min = p.row_lo[wrow0 < S ? wrow0 : S - 1];
        wave_lo_max = p.row_lo[(wrow0 + 31 < S ? wrow0 + 31 : S - 1)];
        wg_lo_min = p.row_lo[i0];
    }
    const int wave_q_min = wrow0, wave_q_max = wrow0 + 31;
    const int jt_begin = VARLEN ? wg_lo_min / DQ_BN : 0;
    const int last_row = (i0 + DQ_BM - 1 < S ? i0 + DQ_BM - 1 : S - 1);
    const int jt_end = last_row / DQ_BN + 1;

    f32x16 dqacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dqacc[db][r] = 0.f;

    u32x4 kst[4], vst[V_LOADS];
    const int t_kg = tid / KCH, t_c = tid % KCH;
    auto load_tile = [&](int jt) {
        const int j0 = jt * DQ_BN;
        if (tid < TASKS) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int row = j0 + 4 * t_kg + e;
                row = row < S ? row : S - 1;
                kst[e] = *reinterpret_cast<const u32x4*>(kb + (size_t)row * kv_row_stride + 8 * t_c);
            }
        }
#pragma unroll
        for (int u = 0; u < V_LOADS; ++u) {
            const int c = tid + u * kThreads;
            int row = j0 + c / KCH;
            row = row < S ? row : S - 1;
            vst[u] = *reinterpret_cast<const u32x4*>(vb + (size_t)row * kv_row_stride + 8 * (c % KCH));
        }
    };
    auto store_tile = [&]() {
        if (tid < TASKS) {
            u32x2 col[8];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                *reinterpret_cast<u32x4*>(&sm.k[(4 * t_kg + e) * LDR + 8 * t_c]) = kst[e];
            transpose4x8(kst, col);
            const int pos = operand_pos4(t_kg);
#pragma unroll
            for (int dd = 0; dd < 8; ++dd) *reinterpret_cast<u32x2*>(&sm.kt[(8 * t_c + dd) * LDT + pos]) = col[dd];
        }
#pragma unroll
        for (int u = 0; u < V_LOADS; ++u) {
            const int c = tid + u * kThreads;
            *reinterpret_cast<u32x4*>(&sm.v[(c / KCH) * LDR + 8 * (c % KCH)]) = vst[u];
        }
    };

    if (jt_begin < jt_end) load_tile(jt_begin);
    for (int jt = jt_begin; jt < jt_end; ++jt) {
        __syncthreads();
        store_tile();
        __syncthreads();
        if (jt + 1 < jt_end) load_tile(jt + 1);

        const int j0 = jt * DQ_BN;
        bool active = j0 <= wave_q_max;
        if (VARLEN) active = active && (j0 + DQ_BN > wave_lo_min);
        if (!active) continue;

        // ---- S^T = K.Q^T, dP^T = V.dO^T (rows = keys in registers, column = this lane's query) ----
        f32x16 sacc[2], pacc[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) { sacc[nb][r] = 0.f; pacc[nb][r] = 0.f; }
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk) {
                const bf16x8 ak = as_bf16x8(*reinterpret_cast<const u32x4*>(&sm.k[(32 * nb + lo) * LDR + 16 * kk + 8 * hi]));
                sacc[nb] = mfma32(ak, qreg[kk], sacc[nb]);
                const bf16x8 av = as_bf16x8(*reinterpret_cast<const u32x4*>(&sm.v[(32 * nb + lo) * LDR + 16 * kk + 8 * hi]));
                pacc[nb] = mfma32(av, doreg[kk], pacc[nb]);
            }
        }
        bool need_mask = j0 + DQ_BN - 1 > wave_q_min;
        if (VARLEN) need_mask = need_mask || (j0 < wave_lo_max);
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float pij = __builtin_amdgcn_exp2f(sacc[nb][r] * p.scale_log2 - lse2);
                if (need_mask) {
                    const int key = j0 + 32 * nb + 8 * (r / 4) + 4 * hi + (r % 4);
                    bool vis = key <= qrow;
                    if (VARLEN) vis = vis && key >= row_lo;
                    pij = vis ? pij : 0.f;
                }
                pacc[nb][r] = pij * (pacc[nb][r] - delta);
            }
        // ---- dQ^T += K^T . dS^T ----
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const bf16x8 dsb = acc_to_operand(pacc[nb], 8 * c);
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(&sm.kt[(32 * db + lo) * LDT + 16 * (2 * nb + c) + 8 * hi]));
                    dqacc[db] = mfma32(a, dsb, dqacc[db]);
                }
            }
    }

    if (qrow < S) {
        __bf16* out = p.dq + (((size_t)b * S + qrow) * p.Hq + h) * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                u32x2 w;
                w[0] = pack_bf16(dqacc[db][4 * gq + 0] * p.scale, dqacc[db][4 * gq + 1] * p.scale);
                w[1] = pack_bf16(dqacc[db][4 * gq + 2] * p.scale, dqacc[db][4 * gq + 3] * p.scale);
                *reinterpret_cast<u32x2*>(out + 32 * db + 8 * gq + 4 * hi) = w;
            }
    }
}

template <int D, bool VARLEN>
sp_status launch(const AttnArgs& a, hipStream_t st) {
    if (a.stages & SP_BWD_STAGE_DELTA) {
        const int64_t lanes = (int64_t)a.B * a.S * a.Hq * (D / 8);
        const int64_t blocks = (lanes + 255) / 256;
        if (blocks > 0x7fffffff) return SP_ERR_SHAPE;
        hipLaunchKernelGGL((delta_kernel<D>), dim3((unsigned)blocks), dim3(256), 0, st, (const __bf16*)a.o,
                           (const __bf16*)a.dO, a.lse, a.delta, a.lsn, a.dn, a.B, a.S, a.S_pad, a.Hq,
                           1.0f / a.scale);
        if (hipGetLastError() != hipSuccess) return SP_ERR_LAUNCH;
        const int64_t npad = (int64_t)a.B * a.Hq * (a.S_pad - a.S);
        hipLaunchKernelGGL(aux_pad_kernel, dim3((unsigned)((npad + 255) / 256)), dim3(256), 0, st, a.lsn, a.dn,
                           a.B * a.Hq, a.S, a.S_pad);
        if (hipGetLastError() != hipSuccess) return SP_ERR_LAUNCH;
    }
    BwdParams p;
    p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.dO = (const __bf16*)a.dO;
    p.lse = a.lse; p.delta = a.delta;
    p.dq = (__bf16*)a.dq; p.dk = (__bf16*)a.dk; p.dv = (__bf16*)a.dv;
    p.row_lo = a.row_lo; p.row_hi = a.row_hi;
    p.S = a.S; p.Hq = a.Hq; p.Hkv = a.Hkv; p.G = a.Hq / a.Hkv;
    p.scale = a.scale; p.scale_log2 = a.scale * kLog2e;
    if (a.stages & SP_BWD_STAGE_DKDV) {
        const sp_status r = launch_attn_bwd_dkdv(a, st);
        if (r != SP_OK) return r;
    }
    if (a.stages & SP_BWD_STAGE_DQ) {
        p.n_tiles = (a.S + DQ_BM - 1) / DQ_BM;
        dim3 grid(p.n_tiles, a.Hq, a.B);
        hipLaunchKernelGGL((attn_bwd_dq_kernel<D, VARLEN>), grid, dim3(kThreads), 0, st, p);
        if (hipGetLastError() != hipSuccess) return SP_ERR_LAUNCH;
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
