// Causal grouped-query attention, forward, for one device's head shard over
// the full sequence (paper Section 2: every device computes attention locally
// on its heads over the whole context; Section 3.1 challenge 3: causal mask).
//
// One workgroup = 4 waves = 128 query rows of one query head; each wave owns 32
// rows; two workgroups share a CU so one's MFMA phase overlaps the other's
// softmax.  Keys/values stream through LDS in tiles of 64, double-buffered and
// filled by direct global->LDS loads into an unpadded XOR-swizzled layout (no
// staging registers, one barrier per tile).  Per tile and wave:
//   S^T[key, query] = K_tile . Q^T          (MFMA; K from LDS as A, Q resident as B)
//   online softmax in fp32: with queries on the lane axis of the accumulator,
//     a row's maximum and sum are register-local plus one swap between the two
//     wave halves; O is rescaled only when some row's maximum moves
//   O^T[d, query] += V_tile^T . P^T         (MFMA; V^T read from the row-major V
//     tile with transposing LDS reads; the S^T accumulator registers, rounded
//     to bf16, are already a valid B operand)
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;

constexpr int kThreads = 256;
constexpr int BM = 128;  // query rows per workgroup
constexpr int BN = 64;   // keys per tile

struct FwdParams {
    const __bf16* q; const __bf16* k; const __bf16* v;
    __bf16* o; float* lse;
    const int32_t* row_lo;
    int32_t S, Hq, Hkv, G, n_qtiles;
    float scale_log2;  // softmax_scale * log2(e)
};

template <int D, bool VARLEN>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(FwdParams p) {
    constexpr int TILE = BN * D;  // elements per K or V tile
    // two K and two V tiles (double buffer), unpadded and swizzled, filled by direct global->LDS loads
    __shared__ __attribute__((aligned(1024))) __bf16 ks[2 * TILE];
    __shared__ __attribute__((aligned(1024))) __bf16 vs[2 * TILE];

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

    // LDS byte offsets of this lane's operand reads, tile-invariant
    int koff[D / 16];  // K row-major operand: row 32*nb + lo (nb adds a constant), chunk 2*kk + hi
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) koff[kk] = tile_off_b128<D>(lo, 2 * kk + hi);
    int voff[2][D / 32];  // V^T operand via transposing reads: rows 16*c + 8*half + 4*hi + (0..3), cols 32*db + 16*(lo/16) + (lo%16)
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
            voff[half][db] = tile_off_tr<D>(8 * half + 4 * hi, 32 * db + 16 * (lo >> 4), lo & 15);

    TileDma<D, BN> dma;
    dma.init(wave, lane);

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_run = -INFINITY;  // running maximum, in log2 units (score * scale * log2 e)
    float l_run = 0.f;        // this lane's share of the running sum

    dma.issue(kb, kv_row_stride, jt_begin * BN, S - 1, ks, wave);
    dma.issue(vb, kv_row_stride, jt_begin * BN, S - 1, vs, wave);
    for (int jt = jt_begin; jt < jt_end; ++jt) {
        const int buf = (jt - jt_begin) & 1;
        wait_vmem();      // this wave's part of tile jt is in LDS
        __syncthreads();  // ... and everybody else's; everybody is also done reading tile jt-1
        if (jt + 1 < jt_end) {
            dma.issue(kb, kv_row_stride, (jt + 1) * BN, S - 1, ks + (buf ^ 1) * TILE, wave);
            dma.issue(vb, kv_row_stride, (jt + 1) * BN, S - 1, vs + (buf ^ 1) * TILE, wave);
        }
        const char* kt = reinterpret_cast<const char*>(ks + buf * TILE);
        const char* vt = reinterpret_cast<const char*>(vs + buf * TILE);

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
                const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(kt + koff[kk] + nb * (32 * D * 2)));
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
        mx = fmaxf(mx, xhalf(mx)) * p.scale_log2;
        // O is rescaled only on tiles where some row of the wave raises its maximum (a few
        // percent of the tiles at long sequence length).  The reference stays the exact row
        // maximum, so the dominant weight of a peaked row is exactly 1 before bf16 rounding.
        if (__builtin_amdgcn_ballot_w64(mx > m_run) != 0) {
            const float m_new = fmaxf(m_run, mx);
            const float m_sub = (m_new == -INFINITY) ? 0.f : m_new;  // fully masked so far
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_sub);
            l_run *= alpha;
            m_run = m_new;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        }
        const float m_sub = (m_run == -INFINITY) ? 0.f : m_run;
        float psum = 0.f;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float e = __builtin_amdgcn_exp2f(sacc[nb][r] * p.scale_log2 - m_sub);
                sacc[nb][r] = e;
                psum += e;
            }
        l_run += psum;
        // ---- O^T += V^T . P^T, 16 keys per step ----
#pragma unroll
        for (int c = 0; c < BN / 16; ++c) {
            const bf16x8 pb = acc_to_operand(sacc[c / 2], 8 * (c % 2));
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const s16x4 v0 = lds_read_tr16(vt + voff[0][db] + c * (16 * D * 2));
                const s16x4 v1 = lds_read_tr16(vt + voff[1][db] + c * (16 * D * 2));
                const s16x8 a8 = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                oacc[db] = mfma32(__builtin_bit_cast(bf16x8, a8), pb, oacc[db]);
            }
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
