// dQ of causal grouped-query attention (paper Section 3.1: the rewritten graph
// must stay correct in the backward pass; Section 4.4: the backward is where
// recomputation under activation checkpointing is paid).
//
//   dQ_i = scale * sum_{j<=i} dS_ij k_j,   dS_ij = P_ij (dO_i.v_j - Delta_i),
//   P_ij = exp(scale * q_i.k_j - LSE_i)
//
// One workgroup = 4 waves = 256 query rows of one query head, one wave per SIMD;
// a wave owns 64 rows (two 32-row blocks): their Q and dO stay in registers as
// MFMA B operands and their dQ lives in accumulator registers that only MFMAs
// touch.  K/V tiles of 64 keys stream through LDS (direct global->LDS loads,
// double-buffered, XOR-swizzled); every operand fetched from LDS feeds two
// MFMAs, one per row block.  Per 32-key step and wave:
//   S^T = K.Q^T, dP^T = V.dO^T          (keys on the register axis, one query per
//        lane, so LSE and Delta are per-lane scalars; accumulators pinned to
//        vector registers where the arithmetic reads them)
//   dS = exp2(S*scale*log2e - LSE*log2e) * (dP - Delta)   (fp32 VALU, then bf16)
//   dQ^T += K^T.dS^T                    (K^T from transposing LDS reads; the dS^T
//        accumulator tile is already a valid B operand)
// All LDS operand reads are asynchronous with explicit partial waits.
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int RPW = 64;           // query rows per wave
constexpr int BM = RPW * kWaves;  // query rows per workgroup
constexpr int BN = 64;            // keys per streamed tile (two 32-key steps)

struct DqParams {
    const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* dO;
    const float* lse; const float* delta;
    __bf16* dq;
    const int32_t* row_lo;
    int32_t S, Hq, Hkv, G, n_qtiles;
    float scale, scale_log2;
};

template <int D, bool VARLEN>
__global__ __launch_bounds__(kThreads) void attn_bwd_dq_kernel(DqParams p) {
    constexpr int TILE = BN * D;
    constexpr int NKK = D / 16;
    constexpr int NDB = D / 32;
    __shared__ __attribute__((aligned(1024))) __bf16 ks[2 * TILE];
    __shared__ __attribute__((aligned(1024))) __bf16 vs[2 * TILE];

    const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // heads vary fastest (they share K/V tiles), query tiles from the last (longest) to the first
    const int h = blockIdx.x % p.Hq;
    const int qt = p.n_qtiles - 1 - (int)(blockIdx.x / p.Hq);
    const int b = blockIdx.y, g = h / p.G;
    const int S = p.S;
    const size_t q_row_stride = (size_t)p.Hq * D, kv_row_stride = (size_t)p.Hkv * D;
    const __bf16* qb_ = p.q + ((size_t)b * S * p.Hq + h) * D;
    const __bf16* dob = p.dO + ((size_t)b * S * p.Hq + h) * D;
    const __bf16* kb = p.k + ((size_t)b * S * p.Hkv + g) * D;
    const __bf16* vb = p.v + ((size_t)b * S * p.Hkv + g) * D;

    const int i0 = qt * BM;
    const int wrow0 = i0 + RPW * wave;  // first row of this wave

    bf16x8 qreg[2][NKK], doreg[2][NKK];
    int qrow[2], row_lo[2];
    float lse2[2], delta[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        qrow[qb] = wrow0 + 32 * qb + lo;
        const int rc = qrow[qb] < S ? qrow[qb] : S - 1;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            qreg[qb][kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(qb_ + (size_t)rc * q_row_stride + 16 * kk + 8 * hi));
            doreg[qb][kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(dob + (size_t)rc * q_row_stride + 16 * kk + 8 * hi));
        }
        lse2[qb] = p.lse[((size_t)b * p.Hq + h) * S + rc] * kLog2e;
        delta[qb] = p.delta[((size_t)b * p.Hq + h) * S + rc];
        row_lo[qb] = VARLEN ? p.row_lo[rc] : 0;
    }
    int wave_lo_min = 0, wave_lo_max = 0, wg_lo_min = 0;
    if (VARLEN) {
        wave_lo_min = __builtin_amdgcn_readfirstlane(p.row_lo[wrow0 < S ? wrow0 : S - 1]);
        wave_lo_max = __builtin_amdgcn_readfirstlane(p.row_lo[(wrow0 + RPW - 1 < S ? wrow0 + RPW - 1 : S - 1)]);
        wg_lo_min = __builtin_amdgcn_readfirstlane(p.row_lo[i0]);
    }
    const int wave_q_min = wrow0, wave_q_max = wrow0 + RPW - 1;
    const int jt_begin = VARLEN ? wg_lo_min / BN : 0;
    const int last_row = (i0 + BM - 1 < S ? i0 + BM - 1 : S - 1);
    const int jt_end = last_row / BN + 1;  // exclusive

    f32x16 dqacc[2][NDB];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) dqacc[qb][db][r] = 0.f;

    int roff[NKK];  // row-major operand (K, V rows): row lo (+32 per step), chunk 2*kk + hi
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) roff[kk] = tile_off_b128<D>(lo, 2 * kk + hi);
    int toff[2][NDB];  // K^T operand: rows 16*c + 8*half + 4*hi + (0..3), cols 32*db + 16*(lo/16) + lo%16
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
            toff[half][db] = tile_off_tr<D>(8 * half + 4 * hi, 32 * db + 16 * (lo >> 4), lo & 15);

    TileDma<D, BN, kWaves> dma;
    dma.init(wave, lane, kv_row_stride);

    // one 32-key step: keys j0 .. j0+31 = rows 32*nb.. of the tile in buffer `buf`
    auto step32 = [&](int buf, int nb, int j0) __attribute__((always_inline)) {
        bool active = j0 <= wave_q_max;
        if (VARLEN) active = active && (j0 + 32 > wave_lo_min);
        if (!active) return;
        const uint32_t ka = lds_addr(ks + buf * TILE) + nb * (32 * D * 2);
        const uint32_t va = lds_addr(vs + buf * TILE) + nb * (32 * D * 2);

        // ---- stage 1: S^T and dP^T for both row blocks ----
        u32x4 ak[NKK], av[NKK];
        constexpr int kAhead = 2;
        auto load1 = [&](auto KK) __attribute__((always_inline)) {
            constexpr int kk = decltype(KK)::value;
            ak[kk] = lds_async_b128<0>(ka + roff[kk]);
            av[kk] = lds_async_b128<0>(va + roff[kk]);
        };
        static_for<0, kAhead>([&](auto I) { load1(I); });
        f32x16 sacc[2], pacc[2];
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, NKK>([&](auto KK) {
            constexpr int kk = decltype(KK)::value;
            if constexpr (kk + kAhead < NKK) load1(std::integral_constant<int, kk + kAhead>{});
            constexpr int m2 = 2 * ((kk + kAhead < NKK ? kAhead : NKK - 1 - kk));  // reads of later groups in flight
            lds_wait<m2 + 1>(ak[kk]);
            if constexpr (kk == 0) {
                mfma32_v0(sacc[0], ak[kk], qreg[0][kk]);
                mfma32_v0(sacc[1], ak[kk], qreg[1][kk]);
            } else {
                mfma32_v(sacc[0], ak[kk], qreg[0][kk]);
                mfma32_v(sacc[1], ak[kk], qreg[1][kk]);
            }
            lds_wait<m2>(av[kk]);
            if constexpr (kk == 0) {
                mfma32_v0(pacc[0], av[kk], doreg[0][kk]);
                mfma32_v0(pacc[1], av[kk], doreg[1][kk]);
            } else {
                mfma32_v(pacc[0], av[kk], doreg[0][kk]);
                mfma32_v(pacc[1], av[kk], doreg[1][kk]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        mfma_results_ready(sacc[0], sacc[1], pacc[0], pacc[1]);

        // ---- stage 2: dS = P (dP - Delta) ----
        bool need_mask = j0 + 31 > wave_q_min;
        if (VARLEN) need_mask = need_mask || (j0 < wave_lo_max);
        u32x4 dsp[2][2];  // bf16 B operands: [row block][16-key step]
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                float p0 = __builtin_amdgcn_exp2f(sacc[qb][r] * p.scale_log2 - lse2[qb]);
                float p1 = __builtin_amdgcn_exp2f(sacc[qb][r + 1] * p.scale_log2 - lse2[qb]);
                if (need_mask) {
                    const int key0 = j0 + 8 * (r / 4) + 4 * hi + (r % 4);
                    bool v0 = key0 <= qrow[qb], v1 = key0 + 1 <= qrow[qb];
                    if (VARLEN) { v0 = v0 && key0 >= row_lo[qb]; v1 = v1 && key0 + 1 >= row_lo[qb]; }
                    p0 = v0 ? p0 : 0.f;
                    p1 = v1 ? p1 : 0.f;
                }
                const float d0 = p0 * (pacc[qb][r] - delta[qb]), d1 = p1 * (pacc[qb][r + 1] - delta[qb]);
                dsp[qb][r / 8][(r % 8) / 2] = pack_bf16(d0, d1);
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- stage 3: dQ^T += K^T . dS^T ----
        constexpr int N3 = 2 * NDB;  // (16-key step c, d block db)
        constexpr int kAhead3 = 2;
        u32x2 t0[N3], t1[N3];
        auto load3 = [&](auto T) __attribute__((always_inline)) {
            constexpr int t = decltype(T)::value, c = t / NDB, db = t % NDB;
            t0[t] = lds_async_tr16<c * (16 * D * 2)>(ka + toff[0][db]);
            t1[t] = lds_async_tr16<c * (16 * D * 2)>(ka + toff[1][db]);
        };
        static_for<0, kAhead3>([&](auto T) { load3(T); });
        static_for<0, N3>([&](auto T) {
            constexpr int t = decltype(T)::value, c = t / NDB, db = t % NDB;
            if constexpr (t + kAhead3 < N3) load3(std::integral_constant<int, t + kAhead3>{});
            constexpr int ahead = (t + kAhead3 < N3 ? kAhead3 : N3 - 1 - t);
            lds_wait<2 * ahead>(t0[t], t1[t]);
            const u32x4 kt = {t0[t][0], t0[t][1], t1[t][0], t1[t][1]};
            dqacc[0][db] = mfma32(as_bf16x8(kt), as_bf16x8(dsp[0][c]), dqacc[0][db]);
            dqacc[1][db] = mfma32(as_bf16x8(kt), as_bf16x8(dsp[1][c]), dqacc[1][db]);
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    if (jt_begin < jt_end) {
        dma.issue(kb, jt_begin * BN, S - 1, ks, wave);
        dma.issue(vb, jt_begin * BN, S - 1, vs, wave);
    }
    for (int jt = jt_begin; jt < jt_end; ++jt) {
        const int buf = (jt - jt_begin) & 1;
        wait_vmem();      // this wave's share of tile jt is in LDS
        __syncthreads();  // ... and everybody else's; everybody is done reading the other buffer
        if (jt + 1 < jt_end) {
            dma.issue(kb, (jt + 1) * BN, S - 1, ks + (buf ^ 1) * TILE, wave);
            dma.issue(vb, (jt + 1) * BN, S - 1, vs + (buf ^ 1) * TILE, wave);
        }
        step32(buf, 0, jt * BN);
        step32(buf, 1, jt * BN + 32);
    }

    // ---- write dQ (scaled): accumulator rows = d, column = this lane's query ----
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        if (qrow[qb] < S) {
            __bf16* out = p.dq + (((size_t)b * S + qrow[qb]) * p.Hq + h) * D;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    u32x2 w;
                    w[0] = pack_bf16(dqacc[qb][db][4 * gq + 0] * p.scale, dqacc[qb][db][4 * gq + 1] * p.scale);
                    w[1] = pack_bf16(dqacc[qb][db][4 * gq + 2] * p.scale, dqacc[qb][db][4 * gq + 3] * p.scale);
                    *reinterpret_cast<u32x2*>(out + 32 * db + 8 * gq + 4 * hi) = w;
                }
        }
    }
}

template <int D, bool VARLEN>
sp_status launch(const AttnArgs& a, hipStream_t st) {
    DqParams p;
    p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.dO = (const __bf16*)a.dO;
    p.lse = a.lse; p.delta = a.delta; p.dq = (__bf16*)a.dq; p.row_lo = a.row_lo;
    p.S = a.S; p.Hq = a.Hq; p.Hkv = a.Hkv; p.G = a.Hq / a.Hkv;
    p.n_qtiles = (a.S + BM - 1) / BM;
    p.scale = a.scale; p.scale_log2 = a.scale * kLog2e;
    dim3 grid(p.n_qtiles * a.Hq, a.B);
    hipLaunchKernelGGL((attn_bwd_dq_kernel<D, VARLEN>), grid, dim3(kThreads), 0, st, p);
    return launch_status();
}

}  // namespace

namespace sp {

sp_status launch_attn_bwd_dq(const AttnArgs& a, hipStream_t st) {
    if (a.B > 65535) return SP_ERR_SHAPE;
    const bool varlen = a.row_lo != nullptr;
    if (a.D == 128) return varlen ? launch<128, true>(a, st) : launch<128, false>(a, st);
    if (a.D == 64) return varlen ? launch<64, true>(a, st) : launch<64, false>(a, st);
    return SP_ERR_UNSUPPORTED;
}

}  // namespace sp
