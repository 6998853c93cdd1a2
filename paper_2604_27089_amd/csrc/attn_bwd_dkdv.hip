// dK and dV of causal grouped-query attention (paper Section 3.1: the rewritten
// graph must stay correct in the backward pass; Section 4.4: the backward is
// where recomputation under activation checkpointing is paid).
//
//   dV_j = sum_{a in group} sum_{i>=j} P_ij dO_i
//   dK_j = scale * sum_{a in group} sum_{i>=j} dS_ij q_i,   dS_ij = P_ij (dO_i.v_j - Delta_i)
//
// One workgroup = 4 waves = 256 keys of one KV head, one wave per SIMD; a wave
// owns 64 keys (two 32-key blocks): their K stays in registers as MFMA B operand,
// their V sits in LDS for the whole kernel, and their dK, dV live in 256
// accumulator registers that only MFMAs touch.  A streamed operand fetched from
// LDS feeds two MFMAs (one per key block), which keeps the LDS traffic per flop
// well below what a 32-key wave would need.
//
// The Q/dO rows of the G query heads of the group stream through LDS in tiles
// of 64 rows (direct global->LDS loads, double-buffered, XOR-swizzled), from the
// last row down to the diagonal so that co-resident workgroups read the same
// rows at the same time.  Per 32-row step and wave:
//   S' = Q.K^T - LSE/scale, dP' = dO.V^T - Delta   (the subtractions ride in the
//        accumulator initial value, fetched per row from LDS)
//   P = exp2(S' * scale*log2e), dS = P * dP'       (fp32 VALU, then bf16)
//   dV += P^T.dO, dK += dS^T.Q                     (P and dS accumulator tiles are
//        already valid A operands; dO^T and Q^T come from transposing LDS reads)
// All LDS operand reads are asynchronous with explicit partial waits.
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int KPW = 64;            // keys per wave
constexpr int BNK = KPW * kWaves;  // keys per workgroup
constexpr int BMQ = 64;            // query rows per streamed tile (two 32-row steps)

struct DkdvParams {
    const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* dO;
    const float* lsn;  // -LSE/scale, [B, Hq, S_pad]
    const float* dn;   // -Delta,     [B, Hq, S_pad]
    __bf16* dk; __bf16* dv;
    const int32_t* row_hi;
    int32_t S, S_pad, Hq, Hkv, G, n_ktiles;
    float scale, scale_log2;
};

template <int N>
__device__ __forceinline__ void lds_wait4(u32x4& a, u32x4& b, u32x4& c, u32x4& d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}

template <int D, bool VARLEN>
__global__ __launch_bounds__(kThreads) void attn_bwd_dkdv_kernel(DkdvParams p) {
    constexpr int TILE = BMQ * D;
    constexpr int NKK = D / 16;  // contraction steps over the head dim
    constexpr int NDB = D / 32;  // 32-wide blocks of the head dim
    __shared__ __attribute__((aligned(1024))) __bf16 qs[2 * TILE];
    __shared__ __attribute__((aligned(1024))) __bf16 dos[2 * TILE];
    __shared__ __attribute__((aligned(1024))) __bf16 vs[BNK * D];  // V of the workgroup's keys, resident
    __shared__ __attribute__((aligned(256))) float lss[2 * BMQ];
    __shared__ __attribute__((aligned(256))) float dns[2 * BMQ];

    const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jt = blockIdx.x;  // earliest key tiles (most rows to visit) first
    const int g = blockIdx.y, b = blockIdx.z;
    const int S = p.S;
    const size_t q_row_stride = (size_t)p.Hq * D, kv_row_stride = (size_t)p.Hkv * D;
    const __bf16* kb = p.k + ((size_t)b * S * p.Hkv + g) * D;
    const __bf16* vb = p.v + ((size_t)b * S * p.Hkv + g) * D;

    const int j0 = jt * BNK;
    const int wkey0 = j0 + KPW * wave;  // first key of this wave

    // resident B operand: K^T columns of this lane's two keys
    bf16x8 kreg[2][NKK];
    int key_hi[2];  // one past the last query row that may see the key
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk) {
        const int key = wkey0 + 32 * kbk + lo;
        const int key_c = key < S ? key : S - 1;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            kreg[kbk][kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(kb + (size_t)key_c * kv_row_stride + 16 * kk + 8 * hi));
        }
        key_hi[kbk] = VARLEN ? p.row_hi[key_c] : S;
    }
    int wave_hi_min = S, wave_hi_max = S, wg_hi_max = S;
    if (VARLEN) {
        wave_hi_min = __builtin_amdgcn_readfirstlane(p.row_hi[(wkey0 < S ? wkey0 : S - 1)]);
        wave_hi_max = __builtin_amdgcn_readfirstlane(p.row_hi[(wkey0 + KPW - 1 < S ? wkey0 + KPW - 1 : S - 1)]);
        wg_hi_max = __builtin_amdgcn_readfirstlane(p.row_hi[(j0 + BNK - 1 < S ? j0 + BNK - 1 : S - 1)]);
    }

    f32x16 dkacc[2][NDB], dvacc[2][NDB];
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) { dkacc[kbk][db][r] = 0.f; dvacc[kbk][db][r] = 0.f; }

    // tile-invariant LDS byte offsets of this lane's operand reads
    int roff[NKK];  // row-major operand (Q, dO rows): row lo (+32 per step), chunk 2*kk + hi
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) roff[kk] = tile_off_b128<D>(lo, 2 * kk + hi);
    int toff[2][NDB];  // transposed operand (Q^T, dO^T): rows 16*c + 8*half + 4*hi + (0..3), cols 32*db + 16*(lo/16) + lo%16
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
            toff[half][db] = tile_off_tr<D>(8 * half + 4 * hi, 32 * db + 16 * (lo >> 4), lo & 15);
    const int aoff = 16 * hi;  // per-row scalars: rows 8*g + 4*hi .. +3 of a 32-row step

    TileDma<D, BMQ, kWaves> dma;
    dma.init(wave, lane, q_row_stride);
    {
        // V rows j0 .. j0+255 -> LDS once (rows past the end re-read the last row; never used unmasked)
        TileDma<D, BNK, kWaves> vdma;
        vdma.init(wave, lane, kv_row_stride);
        vdma.issue(vb, j0, S - 1, vs, wave);
    }

    const int it_begin = j0 / BMQ;                    // tile holding the first key's own row
    const int it_end = (wg_hi_max + BMQ - 1) / BMQ;   // exclusive
    const int n_it = it_end - it_begin;
    const int total = n_it * p.G;                     // (head in group, row tile) pairs, rows descending

    auto issue_tile = [&](int step, int buf) __attribute__((always_inline)) {
        const int a = g * p.G + step / n_it;
        const int i0 = (it_end - 1 - step % n_it) * BMQ;
        const __bf16* qb = p.q + ((size_t)b * S * p.Hq + a) * D;
        const __bf16* dob = p.dO + ((size_t)b * S * p.Hq + a) * D;
        dma.issue(qb, i0, S - 1, qs + buf * TILE, wave);
        dma.issue(dob, i0, S - 1, dos + buf * TILE, wave);
        if (wave == 0 && lane < 16) {  // 64 floats = 16 lanes x 16 bytes; the arrays are padded past S
            const size_t base = ((size_t)b * p.Hq + a) * p.S_pad + i0;
            dma16(p.lsn + base + 4 * lane, lss + buf * BMQ);
            dma16(p.dn + base + 4 * lane, dns + buf * BMQ);
        }
    };

    // one 32-row step: rows q0 .. q0+31, operands in buffer `buf`, rows 32*mb.. of the tile
    auto step32 = [&](int buf, int mb, int q0) __attribute__((always_inline)) {
        bool active = q0 + 31 >= wkey0 && q0 < S;
        if (VARLEN) active = active && q0 < wave_hi_max;
        if (!active) return;
        const uint32_t qa = lds_addr(qs + buf * TILE) + mb * (32 * D * 2);
        const uint32_t da = lds_addr(dos + buf * TILE) + mb * (32 * D * 2);
        const uint32_t la = lds_addr(lss + buf * BMQ) + mb * 128 + aoff;
        const uint32_t na = lds_addr(dns + buf * BMQ) + mb * 128 + aoff;
        const uint32_t va = lds_addr(vs) + wave * (KPW * D * 2);             // this wave's 64 V rows
        const uint32_t qta = lds_addr(qs + buf * TILE) + mb * (32 * D * 2);   // same rows, transposing reads
        const uint32_t dta = lds_addr(dos + buf * TILE) + mb * (32 * D * 2);

        // ---- stage 1: S' and dP' for both key blocks ----
        // The four accumulators are seeded straight from LDS with -LSE/scale resp. -Delta of the
        // 16 rows a lane holds (one set of reads per accumulator, so no register copies), then
        // accumulate in vector registers where the softmax arithmetic reads them.
        u32x4 seed[4][4];  // [S0, S1, dP0, dP1][row quad]
        static_for<0, 4>([&](auto G4) { seed[0][G4] = lds_async_b128<32 * decltype(G4)::value>(la); });
        static_for<0, 4>([&](auto G4) { seed[1][G4] = lds_async_b128<32 * decltype(G4)::value>(la); });
        static_for<0, 4>([&](auto G4) { seed[2][G4] = lds_async_b128<32 * decltype(G4)::value>(na); });
        static_for<0, 4>([&](auto G4) { seed[3][G4] = lds_async_b128<32 * decltype(G4)::value>(na); });
        static_for<0, 4>([&](auto A) { lds_wait4<4 * (3 - decltype(A)::value)>(seed[A][0], seed[A][1], seed[A][2], seed[A][3]); });
        f32x16 sacc[2], pacc[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            // (go through scalars: bit-casting a vector element expression directly is not reliable)
            const uint32_t u0 = seed[0][r / 4][r % 4], u1 = seed[1][r / 4][r % 4];
            const uint32_t u2 = seed[2][r / 4][r % 4], u3 = seed[3][r / 4][r % 4];
            sacc[0][r] = __uint_as_float(u0); sacc[1][r] = __uint_as_float(u1);
            pacc[0][r] = __uint_as_float(u2); pacc[1][r] = __uint_as_float(u3);
        }
        u32x4 aq[NKK], ad[NKK], bv0[NKK], bv1[NKK];
        constexpr int kAhead = 2;
        auto load1 = [&](auto KK) __attribute__((always_inline)) {
            constexpr int kk = decltype(KK)::value;
            aq[kk] = lds_async_b128<0>(qa + roff[kk]);
            ad[kk] = lds_async_b128<0>(da + roff[kk]);
            bv0[kk] = lds_async_b128<0>(va + roff[kk]);
            bv1[kk] = lds_async_b128<32 * D * 2>(va + roff[kk]);
        };
        static_for<0, kAhead>([&](auto I) { load1(I); });
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, NKK>([&](auto KK) {
            constexpr int kk = decltype(KK)::value;
            if constexpr (kk + kAhead < NKK) load1(std::integral_constant<int, kk + kAhead>{});
            constexpr int m4 = 4 * ((kk + kAhead < NKK ? kAhead : NKK - 1 - kk));  // reads of later groups in flight
            lds_wait<m4 + 3>(aq[kk]);
            mfma32_v(sacc[0], aq[kk], kreg[0][kk]);
            mfma32_v(sacc[1], aq[kk], kreg[1][kk]);
            lds_wait<m4 + 1>(ad[kk]);
            lds_wait<m4 + 1>(bv0[kk]);
            mfma32_v(pacc[0], ad[kk], bv0[kk]);
            lds_wait<m4>(bv1[kk]);
            mfma32_v(pacc[1], ad[kk], bv1[kk]);
            __builtin_amdgcn_sched_barrier(0);
        });
        mfma_results_ready(sacc[0], sacc[1], pacc[0], pacc[1]);

        constexpr int N3 = 2 * NDB;  // stage-3 iterations: (16-row step c, d block db)
        constexpr int kAhead3 = 2;
        u32x2 bd0[N3], bd1[N3], bq0[N3], bq1[N3];
        auto load3 = [&](auto T) __attribute__((always_inline)) {
            constexpr int t = decltype(T)::value, c = t / NDB, db = t % NDB;
            bd0[t] = lds_async_tr16<c * (16 * D * 2)>(dta + toff[0][db]);
            bd1[t] = lds_async_tr16<c * (16 * D * 2)>(dta + toff[1][db]);
            bq0[t] = lds_async_tr16<c * (16 * D * 2)>(qta + toff[0][db]);
            bq1[t] = lds_async_tr16<c * (16 * D * 2)>(qta + toff[1][db]);
        };

        // ---- stage 2: P = exp2(S' * scale*log2e), dS = P * dP' ----
        bool need_mask = q0 < wkey0 + KPW - 1 || q0 + 31 >= wave_hi_min;
        u32x4 pp[2][2], dsp[2][2];  // bf16 A operands: [key block][16-row step]
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk) {
            const int key = wkey0 + 32 * kbk + lo;
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                float p0 = __builtin_amdgcn_exp2f(sacc[kbk][r] * p.scale_log2);
                float p1 = __builtin_amdgcn_exp2f(sacc[kbk][r + 1] * p.scale_log2);
                if (need_mask) {
                    const int qr0 = q0 + 8 * (r / 4) + 4 * hi + (r % 4);
                    p0 = (qr0 >= key && qr0 < key_hi[kbk]) ? p0 : 0.f;
                    p1 = (qr0 + 1 >= key && qr0 + 1 < key_hi[kbk]) ? p1 : 0.f;
                }
                const float d0 = p0 * pacc[kbk][r], d1 = p1 * pacc[kbk][r + 1];
                pp[kbk][r / 8][(r % 8) / 2] = pack_bf16(p0, p1);
                dsp[kbk][r / 8][(r % 8) / 2] = pack_bf16(d0, d1);
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- stage 3: dV += P^T.dO, dK += dS^T.Q ----
        static_for<0, kAhead3>([&](auto T) { load3(T); });
        static_for<0, N3>([&](auto T) {
            constexpr int t = decltype(T)::value, c = t / NDB, db = t % NDB;
            if constexpr (t + kAhead3 < N3) load3(std::integral_constant<int, t + kAhead3>{});
            constexpr int ahead = (t + kAhead3 < N3 ? kAhead3 : N3 - 1 - t);  // younger iterations in flight
            lds_wait<4 * ahead + 2>(bd0[t], bd1[t]);
            const u32x4 bdo = {bd0[t][0], bd0[t][1], bd1[t][0], bd1[t][1]};
            dvacc[0][db] = mfma32(as_bf16x8(pp[0][c]), as_bf16x8(bdo), dvacc[0][db]);
            dvacc[1][db] = mfma32(as_bf16x8(pp[1][c]), as_bf16x8(bdo), dvacc[1][db]);
            lds_wait<4 * ahead>(bq0[t], bq1[t]);
            const u32x4 bqt = {bq0[t][0], bq0[t][1], bq1[t][0], bq1[t][1]};
            dkacc[0][db] = mfma32(as_bf16x8(dsp[0][c]), as_bf16x8(bqt), dkacc[0][db]);
            dkacc[1][db] = mfma32(as_bf16x8(dsp[1][c]), as_bf16x8(bqt), dkacc[1][db]);
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    if (total > 0) issue_tile(0, 0);
    for (int step = 0; step < total; ++step) {
        const int buf = step & 1;
        wait_vmem();      // this wave's share of tile `step` is in LDS
        __syncthreads();  // ... and everybody else's; everybody is done reading the other buffer
        if (step + 1 < total) issue_tile(step + 1, buf ^ 1);
        const int i0 = (it_end - 1 - step % n_it) * BMQ;
        step32(buf, 1, i0 + 32);
        step32(buf, 0, i0);
    }

    // ---- write dK (scaled) and dV: accumulator rows = keys, column = d ----
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int krow = wkey0 + 32 * kbk + 8 * (r / 4) + 4 * hi + (r % 4);
                if (krow < S) {
                    const size_t off = (((size_t)b * S + krow) * p.Hkv + g) * D + 32 * db + lo;
                    p.dk[off] = (__bf16)(dkacc[kbk][db][r] * p.scale);
                    p.dv[off] = (__bf16)dvacc[kbk][db][r];
                }
            }
}

template <int D, bool VARLEN>
sp_status launch(const AttnArgs& a, hipStream_t st) {
    DkdvParams p;
    p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.dO = (const __bf16*)a.dO;
    p.lsn = a.lsn; p.dn = a.dn; p.dk = (__bf16*)a.dk; p.dv = (__bf16*)a.dv; p.row_hi = a.row_hi;
    p.S = a.S; p.S_pad = a.S_pad; p.Hq = a.Hq; p.Hkv = a.Hkv; p.G = a.Hq / a.Hkv;
    p.n_ktiles = (a.S + BNK - 1) / BNK;
    p.scale = a.scale; p.scale_log2 = a.scale * kLog2e;
    dim3 grid(p.n_ktiles, a.Hkv, a.B);
    hipLaunchKernelGGL((attn_bwd_dkdv_kernel<D, VARLEN>), grid, dim3(kThreads), 0, st, p);
    return launch_status();
}

}  // namespace

namespace sp {

sp_status launch_attn_bwd_dkdv(const AttnArgs& a, hipStream_t st) {
    if (a.Hkv > 65535 || a.B > 65535) return SP_ERR_SHAPE;
    const bool varlen = a.row_lo != nullptr;
    if (a.D == 128) return varlen ? launch<128, true>(a, st) : launch<128, false>(a, st);
    if (a.D == 64) return varlen ? launch<64, true>(a, st) : launch<64, false>(a, st);
    return SP_ERR_UNSUPPORTED;
}

}  // namespace sp
