// Causal grouped-query attention, forward, for one device's head shard over
// the full sequence (paper Section 2: every device computes attention locally
// on its heads over the whole context; Section 3.1 challenge 3: causal mask).
//
// One workgroup = 4 waves = 128 query rows of one query head; each wave owns 32
// rows.  Keys/values stream through LDS in tiles of 64.  Per tile and wave:
//   S^T[key, query] = K_tile . Q^T          (MFMA; K from LDS as A, Q resident as B)
//   online softmax in fp32: with queries on the lane axis of the accumulator,
//     a row's maximum and sum are register-local plus one swap between the two
//     wave halves
//   O^T[d, query] += V_tile^T . P^T         (MFMA; V^T from LDS as A, the S^T
//     accumulator registers, rounded to bf16, are already a valid B operand)
// V is transposed once, on its way into LDS (4x8 register transpose, 8-byte
// LDS stores in operand order).  The next tile's global loads are issued before
// the current tile's arithmetic and parked in registers.
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;

constexpr int kThreads = 256;
constexpr int BM = 128;  // query rows per workgroup
constexpr int BN = 64;   // keys per tile

template <int D>
struct FwdSmem {
    static constexpr int LDK = D + 8;   // K tile row stride (bf16), padded
    static constexpr int LDV = BN + 8;  // V^T tile row stride (bf16), padded
    __bf16 k[BN * LDK];
    __bf16 vt[D * LDV];
};

struct FwdParams {
    const __bf16* q; const __bf16* k; const __bf16* v;
    __bf16* o; float* lse;
    const int32_t* row_lo;
    int32_t S, Hq, Hkv, G, n_qtiles;
    float scale_log2;  // softmax_scale * log2(e)
};

template <int D, bool VARLEN>
__global__ __launch_bounds__(kThreads) void attn_fwd_kernel(FwdParams p) {
    constexpr int KCH = D / 8;                       // 16-byte chunks per row
    constexpr int K_LOADS = BN * KCH / kThreads;     // K chunks per thread per tile
    constexpr int V_TASKS = (BN / 4) * KCH;          // 4-key x 8-dim transposing tasks
    constexpr int LDK = FwdSmem<D>::LDK, LDV = FwdSmem<D>::LDV;
    __shared__ FwdSmem<D> sm;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
    // heaviest (latest) query tiles first
    const int qt = p.n_qtiles - 1 - (int)(blockIdx.x);
    const int h = blockIdx.y, b = blockIdx.z, g = h / p.G;
    const int S = p.S;
    const size_t q_row_stride = (size_t)p.Hq * D, kv_row_stride = (size_t)p.Hkv * D;
    const __bf16* qb = p.q + ((size_t)b * S * p.Hq + h) * D;
    const __bf16* kb = p.k + ((size_t)b * S * p.Hkv + g) * D;
    const __bf16* vb = p.v + ((size_t)b * S * p.Hkv + g) * D;

    const int i0 = qt * BM;
    const int wrow0 = i0 + 32 * wave;            // first row of this wave
    const int qrow = wrow0 + lo;                 // this lane's query row
    const int qrow_c = qrow < S ? qrow : S - 1;  // clamped for loads

    // Q^T operand, resident: qreg[kk] = Q[qrow][16*kk + 8*hi .. +7]
    bf16x8 qreg[D / 16];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
        qreg[kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(qb + (size_t)qrow_c * q_row_stride + 16 * kk + 8 * hi));

    int row_lo = 0, wave_lo_min = 0, wave_lo_max = 0, wg_lo_min = 0;
    if (VARLEN) {
        row_lo = p.row_lo[qrow_c];
        const int last = (wrow0 + 31 < S ? wrow0 + 31 : S - 1);
        wave_lo_min = p.row_lo[wrow0 < S ? wrow0 : S - 1];
        wave_lo_max = p.row_lo[last];
        wg_lo_min = p.row_lo[i0];
    }
    const int wave_q_min = wrow0, wave_q_max = wrow0 + 31;

    const int jt_begin = VARLEN ? wg_lo_min / BN : 0;
    const int last_row = (i0 + BM - 1 < S ? i0 + BM - 1 : S - 1);
    const int jt_end = last_row / BN + 1;  // exclusive

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_run = -INFINITY;  // running maximum, in log2 units (score * scale * log2 e)
    float l_run = 0.f;        // this lane's share of the running sum

    // ---- global -> register staging of one K/V tile ----
    u32x4 kst[K_LOADS];
    u32x4 vst[4];
    const int v_kg = tid / KCH, v_c = tid % KCH;  // transposing task of this thread
    auto load_tile = [&](int jt) {
        const int j0 = jt * BN;
#pragma unroll
        for (int u = 0; u < K_LOADS; ++u) {
            const int c = tid + u * kThreads;
            int row = j0 + c / KCH;
            row = row < S ? row : S - 1;
            kst[u] = *reinterpret_cast<const u32x4*>(kb + (size_t)row * kv_row_stride + 8 * (c % KCH));
        }
        if (tid < V_TASKS) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int row = j0 + 4 * v_kg + e;
                row = row < S ? row : S - 1;
                vst[e] = *reinterpret_cast<const u32x4*>(vb + (size_t)row * kv_row_stride + 8 * v_c);
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int u = 0; u < K_LOADS; ++u) {
            const int c = tid + u * kThreads;
            *reinterpret_cast<u32x4*>(&sm.k[(c / KCH) * LDK + 8 * (c % KCH)]) = kst[u];
        }
        if (tid < V_TASKS) {
            u32x2 col[8];
            transpose4x8(vst, col);
            const int pos = operand_pos4(v_kg);
#pragma unroll
            for (int dd = 0; dd < 8; ++dd)
                *reinterpret_cast<u32x2*>(&sm.vt[(8 * v_c + dd) * LDV + pos]) = col[dd];
        }
    };

    if (jt_begin < jt_end) load_tile(jt_begin);
    for (int jt = jt_begin; jt < jt_end; ++jt) {
        __syncthreads();  // everyone finished reading the previous tile
        store_tile();
        __syncthreads();
        if (jt + 1 < jt_end) load_tile(jt + 1);

        const int j0 = jt * BN;
        // does this wave have any visible key in the tile?
        bool active = j0 <= wave_q_max;
        if (VARLEN) active = active && (j0 + BN > wave_lo_min);
        if (!active) continue;

        // ---- S^T = K . Q^T ----
        f32x16 sacc[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[nb][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk) {
                const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(&sm.k[(32 * nb + lo) * LDK + 16 * kk + 8 * hi]));
                sacc[nb] = mfma32(a, qreg[kk], sacc[nb]);
            }
        }
        // ---- mask ----
        bool need_mask = j0 + BN - 1 > wave_q_min;
        if (VARLEN) need_mask = need_mask || (j0 < wave_lo_max);
        if (need_mask) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = j0 + 32 * nb + 8 * (r / 4) + 4 * hi + (r % 4);
                    bool vis = key <= qrow;
                    if (VARLEN) vis = vis && key >= row_lo;
                    if (!vis) sacc[nb][r] = -INFINITY;
                }
        }
        // ---- online softmax (log2 domain) ----
        float mx = sacc[0][0];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[nb][r]);
        mx = fmaxf(mx, xhalf(mx));
        const float m_new = fmaxf(m_run, mx * p.scale_log2);
        const float m_sub = (m_new == -INFINITY) ? 0.f : m_new;  // fully masked so far
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_sub);
        float psum = 0.f;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float e = __builtin_amdgcn_exp2f(sacc[nb][r] * p.scale_log2 - m_sub);
                sacc[nb][r] = e;
                psum += e;
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        // ---- O^T += V^T . P^T ----
        bf16x8 pb[2][2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int c = 0; c < 2; ++c) pb[nb][c] = acc_to_operand(sacc[nb], 8 * c);
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(&sm.vt[(32 * db + lo) * LDV + 16 * (2 * nb + c) + 8 * hi]));
                    oacc[db] = mfma32(a, pb[nb][c], oacc[db]);
                }
    }

    // ---- epilogue: normalise, write O (bf16) and LSE (natural log) ----
    const float l_tot = l_run + xhalf(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    if (qrow < S) {
        __bf16* orow = p.o + (((size_t)b * S + qrow) * p.Hq + h) * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                u32x2 w;
                w[0] = pack_bf16(oacc[db][4 * gq + 0] * inv, oacc[db][4 * gq + 1] * inv);
                w[1] = pack_bf16(oacc[db][4 * gq + 2] * inv, oacc[db][4 * gq + 3] * inv);
                *reinterpret_cast<u32x2*>(orow + 32 * db + 8 * gq + 4 * hi) = w;
            }
        if (hi == 0) p.lse[((size_t)b * p.Hq + h) * S + qrow] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2;
    }
}

template <int D, bool VARLEN>
sp_status launch(const AttnArgs& a, hipStream_t st) {
    FwdParams p;
    p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v;
    p.o = (__bf16*)a.o; p.lse = a.lse; p.row_lo = a.row_lo;
    p.S = a.S; p.Hq = a.Hq; p.Hkv = a.Hkv; p.G = a.Hq / a.Hkv;
    p.n_qtiles = (a.S + BM - 1) / BM;
    p.scale_log2 = a.scale * kLog2e;
    dim3 grid(p.n_qtiles, a.Hq, a.B), block(kThreads);
    hipLaunchKernelGGL((attn_fwd_kernel<D, VARLEN>), grid, block, 0, st, p);
    return launch_status();
}

}  // namespace

namespace sp {

sp_status launch_attn_fwd(const AttnArgs& a, hipStream_t st) {
    if (a.Hq > 65535 || a.B > 65535) return SP_ERR_SHAPE;
    const bool varlen = a.row_lo != nullptr;
    if (a.D == 128) return varlen ? launch<128, true>(a, st) : launch<128, false>(a, st);
    if (a.D == 64) return varlen ? launch<64, true>(a, st) : launch<64, false>(a, st);
    return SP_ERR_UNSUPPORTED;
}

}  // namespace sp
