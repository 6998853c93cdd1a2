// Causal grouped-query attention, forward, for one device's head shard over
// the full sequence (paper Section 2: every device computes attention locally
// on its heads over the whole context; Section 3.1 challenge 3: causal mask).
// The same kernel serves one step of a ring schedule (Section 4.1: keys and
// values arrive block by block): S query rows against Skv keys, row i seeing
// keys j <= i + off; the plain causal call is Skv = S, off = 0.
//
// One workgroup = 8 waves = 256 query rows of one query head; a wave owns 32
// rows.  Keys/values stream through LDS in tiles of 64, double-buffered and
// filled by direct global->LDS loads into an unpadded XOR-swizzled layout.
// Per tile and wave:
//   S^T[key, query] = K_tile . Q^T          (MFMA; K from LDS as A, Q resident as B)
//   online softmax in fp32: with queries on the lane axis of the accumulator,
//     a row's maximum and sum are register-local plus one swap between the two
//     wave halves; O is rescaled only when some row's maximum moves
//   O^T[d, query] += V_tile^T . P^T         (MFMA; V^T read from the row-major V
//     tile with transposing LDS reads; the S^T accumulator registers, rounded
//     to bf16, are already a valid B operand)
//
// A wave issues in order and a lone wave cannot keep both the matrix pipe and
// the vector ALU busy, so the two waves that share a SIMD (w and w+4) are kept
// in opposite phases: between two workgroup barriers the waves of group A issue
// only matrix work (P.V of the previous tile, then S of the next) while the
// waves of group B run their softmax, and at the next barrier they swap.  Group
// B simply starts one interval late.
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int BM = 32 * kWaves;  // query rows per workgroup
constexpr int BN = 64;           // keys per tile

struct FwdParams {
    const __bf16* q; const __bf16* k; const __bf16* v;
    __bf16* o; float* lse;
    const int32_t* row_lo;
    const int32_t* order;  // packed documents: query tiles in the order workgroups take them (or null)
    RowMap qmap, kvmap;
    int32_t S, Skv, off, Hq, Hkv, G, n_qtiles;  // S query rows, Skv keys; row i sees keys j <= i + off
    float scale_log2;  // softmax_scale * log2(e)
};

template <int D, bool VARLEN>
__global__ __launch_bounds__(kThreads) void attn_fwd_kernel(FwdParams p) {
    constexpr int TILE = BN * D;  // elements per K or V tile
    // Buffer b holds the pair (K tile j, V tile j-1) with j % 2 == b: the two tiles one matrix
    // phase consumes.  Separate arrays, and an interval loop unrolled over the two buffers, so
    // the compiler can tell that reads of one buffer never alias the loads in flight to the other.
    __shared__ __attribute__((aligned(1024))) __bf16 ks0[TILE];
    __shared__ __attribute__((aligned(1024))) __bf16 ks1[TILE];
    __shared__ __attribute__((aligned(1024))) __bf16 vs0[TILE];
    __shared__ __attribute__((aligned(1024))) __bf16 vs1[TILE];

    const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2;  // waves w and w+4 share a SIMD and work in opposite phases
    // Workgroups are dispatched in blockIdx.x order first: heads vary fastest, so the query heads that
    // share a KV head walk the same K/V tiles at the same time, and query tiles go from the last
    // (longest) to the first, which keeps the CUs evenly loaded to the end.
    const int h = blockIdx.x % p.Hq, b = blockIdx.x / p.Hq;
    const int rank = (int)(blockIdx.y + kRankY * blockIdx.z);
    if (rank >= p.n_qtiles) return;  // the last z-slice of a grid of more than kRankY tiles may be ragged
    int qt = p.n_qtiles - 1 - rank;
    if (VARLEN && p.order) {  // longest tile first; the value is clamped so that a bad entry cannot become a wild address
        const int v = __builtin_amdgcn_readfirstlane(p.order[rank]);
        qt = v < 0 ? 0 : (v < p.n_qtiles ? v : p.n_qtiles - 1);
    }
    const int g = h / p.G;
    const int S = p.S, Skv = p.Skv;
    const __bf16* qb = p.q + ((size_t)b * S * p.Hq + h) * D;
    const __bf16* kb = p.k + ((size_t)b * Skv * p.Hkv + g) * D;
    const __bf16* vb = p.v + ((size_t)b * Skv * p.Hkv + g) * D;

    const int i0 = qt * BM;
    const int wrow0 = i0 + 32 * wave;            // first row of this wave
    const int qrow = wrow0 + lo;                 // this lane's query row
    const int qrow_c = qrow < S ? qrow : S - 1;  // clamped for loads

    // Q^T operand, resident: qreg[kk] = Q[qrow][16*kk + 8*hi .. +7]
    bf16x8 qreg[D / 16];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
        qreg[kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(qb + p.qmap.off(qrow_c) + 16 * kk + 8 * hi));

    int row_lo = 0, wave_lo_min = 0, wave_lo_max = 0, wg_lo_min = 0;
    if (VARLEN) {
        row_lo = p.row_lo[qrow_c];
        wave_lo_min = __builtin_amdgcn_readfirstlane(p.row_lo[wrow0 < S ? wrow0 : S - 1]);
        wave_lo_max = __builtin_amdgcn_readfirstlane(p.row_lo[(wrow0 + 31 < S ? wrow0 + 31 : S - 1)]);
        wg_lo_min = __builtin_amdgcn_readfirstlane(p.row_lo[i0]);
    }
    // the last key a row may see: i + off, at most the last key there is
    auto last_key = [&](int row) __attribute__((always_inline)) { return row + p.off < Skv - 1 ? row + p.off : Skv - 1; };
    const int qhi = last_key(qrow);
    const int wave_hi_min = last_key(wrow0), wave_hi_max = last_key(wrow0 + 31);

    const int jt_begin = VARLEN ? wg_lo_min / BN : 0;
    const int last_row = (i0 + BM - 1 < S ? i0 + BM - 1 : S - 1);
    const int T = last_key(last_row) / BN + 1 - jt_begin;  // tiles this workgroup walks (>= 1)

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

    TileDma<D, BN, kWaves> dma;
    dma.init(wave, lane, p.kvmap.row_stride);

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    f32x16 sacc[2];  // S^T of the tile between its matrix phase and its softmax phase
    u32x4 pw[4];     // P^T of the tile, bf16, four MFMA operands (16 keys each)
#pragma unroll
    for (int r = 0; r < 16; ++r) { sacc[0][r] = 0.f; sacc[1][r] = 0.f; }
#pragma unroll
    for (int c = 0; c < 4; ++c) pw[c] = u32x4{0, 0, 0, 0};
    float m_run = -INFINITY;  // running maximum, in log2 units (score * scale * log2 e)
    float l_run = 0.f;        // this lane's share of the running sum

    // does this wave have any visible key in tile j (relative index)?
    auto tile_active = [&](int j) __attribute__((always_inline)) {
        const int j0 = (jt_begin + j) * BN;
        bool active = j0 <= wave_hi_max;
        if (VARLEN) active = active && (j0 + BN > wave_lo_min);
        return active;
    };

    // ---- matrix phase j: O^T += V(j-1)^T . P(j-1)^T, then S(j)^T = K(j) . Q^T ----
    // A wave can pull about one 1 KB operand from LDS per MFMA duration, so the phase is a flat
    // software pipeline: the operand of step i+kAhead is requested right after the MFMA of step i
    // is issued, and the order is pinned so the requests stay ahead of their use.  The wave runs
    // at raised priority while it feeds the matrix pipe.
    auto matrix_phase = [&](const __bf16* kbuf, const __bf16* vbuf, int j) __attribute__((always_inline)) {
        const char* kt = reinterpret_cast<const char*>(kbuf);
        const char* vt = reinterpret_cast<const char*>(vbuf);
        const bool do_pv = j >= 1 && j <= T && tile_active(j - 1);
        const bool do_s = j < T && tile_active(j);
        constexpr int N_PV = (BN / 16) * (D / 32);  // P.V steps: (16-key step c, 32-wide d block db)
        constexpr int N_S = 2 * (D / 16);           // S steps: (kk, 32-key block nb)
        constexpr int kAhead = 3;
        const uint32_t ka = lds_addr(kt), va = lds_addr(vt);
        // operand of P.V step I: V^T rows d = 32*db.., 16 keys of step c (two transposing reads)
        auto load_pv = [&](auto I, u32x2& h0, u32x2& h1) __attribute__((always_inline)) {
            constexpr int c = decltype(I)::value / (D / 32), db = decltype(I)::value % (D / 32);
            h0 = lds_async_tr16<c * (16 * D * 2)>(va + voff[0][db]);
            h1 = lds_async_tr16<c * (16 * D * 2)>(va + voff[1][db]);
        };
        // operand of S step I: K rows 32*nb.., head-dim chunk kk (one 16-byte read)
        auto load_s = [&](auto I) __attribute__((always_inline)) {
            constexpr int kk = decltype(I)::value / 2, nb = decltype(I)::value % 2;
            return lds_async_b128<nb * (32 * D * 2)>(ka + koff[kk]);
        };
        __builtin_amdgcn_s_setprio(2);
        u32x4 kpre[kAhead];  // first S operands, requested while the last P.V steps run
        if (do_pv) {
            u32x2 op0[N_PV], op1[N_PV];
            static_for<0, kAhead>([&](auto I) { load_pv(I, op0[I], op1[I]); });
            __builtin_amdgcn_sched_barrier(0);
            static_for<0, N_PV>([&](auto I) {
                constexpr int i = decltype(I)::value;
                if constexpr (i + kAhead < N_PV) {
                    load_pv(std::integral_constant<int, i + kAhead>{}, op0[i + kAhead], op1[i + kAhead]);
                    lds_wait<2 * kAhead>(op0[i], op1[i]);  // the kAhead younger operands are two reads each
                } else {
                    // tail: the first S operands are requested here (also when no S stage follows:
                    // the read is harmless and keeps this code free of branches around the waits);
                    // younger reads = the remaining P.V operands plus the S operands requested so far
                    kpre[i + kAhead - N_PV] = load_s(std::integral_constant<int, i + kAhead - N_PV>{});
                    lds_wait<2 * (N_PV - 1 - i) + (i + kAhead - N_PV + 1)>(op0[i], op1[i]);
                }
                const u32x4 a = {op0[i][0], op0[i][1], op1[i][0], op1[i][1]};
                oacc[i % (D / 32)] = mfma32(as_bf16x8(a), as_bf16x8(pw[i / (D / 32)]), oacc[i % (D / 32)]);
                __builtin_amdgcn_sched_barrier(0);
            });
            static_for<0, kAhead>([&](auto I) { lds_wait<kAhead - 1 - decltype(I)::value>(kpre[I]); });
        } else {
            static_for<0, kAhead>([&](auto I) { kpre[I] = load_s(I); });
            static_for<0, kAhead>([&](auto I) { lds_wait<kAhead - 1 - decltype(I)::value>(kpre[I]); });
        }
        if (do_s) {
            u32x4 op[N_S];
#pragma unroll
            for (int r = 0; r < 16; ++r) { sacc[0][r] = 0.f; sacc[1][r] = 0.f; }
            static_for<kAhead, 2 * kAhead>([&](auto I) { op[I] = load_s(I); });
            __builtin_amdgcn_sched_barrier(0);
            static_for<0, N_S>([&](auto I) {
                constexpr int i = decltype(I)::value;
                if constexpr (i < kAhead) {
                    // operands fetched (and waited for) before the stage began
                    sacc[i % 2] = mfma32(as_bf16x8(kpre[i]), qreg[i / 2], sacc[i % 2]);
                } else {
                    if constexpr (i + kAhead < N_S) {
                        op[i + kAhead] = load_s(std::integral_constant<int, i + kAhead>{});
                        lds_wait<kAhead>(op[i]);
                    } else {
                        lds_wait<N_S - 1 - i>(op[i]);
                    }
                    sacc[i % 2] = mfma32(as_bf16x8(op[i]), qreg[i / 2], sacc[i % 2]);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        }
        __builtin_amdgcn_s_setprio(0);
    };

    // ---- softmax phase j: mask, running maximum (rescaling O when it moves), weights ----
    auto softmax_phase = [&](int j) __attribute__((always_inline)) {
        if (j < 0 || j >= T || !tile_active(j)) return;
        const int j0 = (jt_begin + j) * BN;
        bool need_mask = j0 + BN - 1 > wave_hi_min;
        if (VARLEN) need_mask = need_mask || (j0 < wave_lo_max);
        if (need_mask) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = j0 + 32 * nb + 8 * (r / 4) + 4 * hi + (r % 4);
                    bool vis = key <= qhi;
                    if (VARLEN) vis = vis && key >= row_lo;
                    if (!vis) sacc[nb][r] = -INFINITY;
                }
        }
        float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(fmaxf(mx, sacc[0][r]), sacc[1][r]);
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
            for (int r = 0; r < 16; r += 2) {
                const float e0 = __builtin_amdgcn_exp2f(sacc[nb][r] * p.scale_log2 - m_sub);
                const float e1 = __builtin_amdgcn_exp2f(sacc[nb][r + 1] * p.scale_log2 - m_sub);
                psum += e0;
                psum += e1;
                pw[2 * nb + r / 8][(r % 8) / 2] = pack_bf16(e0, e1);
            }
        l_run += psum;
    };

    // pair j = (K tile j, V tile j-1) -> the given buffers
    auto issue_pair = [&](__bf16* kbuf, __bf16* vbuf, int j) __attribute__((always_inline)) {
        if (j < T) dma.issue(kb + p.kvmap.off((jt_begin + j) * BN), Skv - 1 - (jt_begin + j) * BN, kbuf, wave);
        if (j >= 1 && j <= T) dma.issue(vb + p.kvmap.off((jt_begin + j - 1) * BN), Skv - 1 - (jt_begin + j - 1) * BN, vbuf, wave);
    };

    issue_pair(ks0, vs0, 0);
    issue_pair(ks1, vs1, 1);
    // Every wave runs  M(0) | S(0) | M(1) | S(1) | ... | M(T)  with a workgroup barrier at each
    // "|"; group B takes one extra barrier first and group A one extra at the end, so that in
    // every interval between two barriers one group is in a matrix phase and the other in a
    // softmax phase.  Interval numbering: group A runs M(j) in interval 2j, group B in 2j+1.
    // Pair j is read in intervals 2j and 2j+1; pair j+2 (same buffer) is issued at the start of
    // interval 2j+2 and waited for before the barrier that opens interval 2j+4.
    wait_vmem();
    __syncthreads();                   // opens interval 0 (pairs 0 and 1 landed)
    if (grp == 1) __syncthreads();     // group B idles through interval 0
    for (int j = 0; j <= T; j += 2) {
        // ---- tile j: buffer 0 ----
        if (grp == 0 && j >= 2) issue_pair(ks1, vs1, j + 1);      // interval 2j: pair j+1 -> buffer 1
        matrix_phase(ks0, vs0, j);
        if (grp == 1) wait_vmem();                                // group B closes odd interval 2j+1
        __syncthreads();
        if (grp == 1) issue_pair(ks0, vs0, j + 2);                // interval 2j+2: pair j+2 -> buffer 0
        softmax_phase(j);
        if (grp == 0) wait_vmem();                                // group A closes odd interval 2j+1
        __syncthreads();
        // ---- tile j+1: buffer 1 ----
        if (grp == 0) issue_pair(ks0, vs0, j + 2);                // interval 2j+2
        matrix_phase(ks1, vs1, j + 1);
        if (grp == 1) wait_vmem();                                // closes interval 2j+3
        __syncthreads();
        if (grp == 1) issue_pair(ks1, vs1, j + 3);                // interval 2j+4: pair j+3 -> buffer 1
        softmax_phase(j + 1);
        if (grp == 0) wait_vmem();                                // closes interval 2j+3
        __syncthreads();
    }
    if (grp == 0) __syncthreads();     // group A matches group B's extra barrier

    // ---- epilogue: normalise, write O (bf16) and LSE (natural log) ----
    const float l_tot = l_run + xhalf(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    if (qrow < S) {
        __bf16* orow = p.o + ((size_t)b * S * p.Hq + h) * D + p.qmap.off(qrow);
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
    p.o = (__bf16*)a.o; p.lse = a.lse; p.row_lo = a.row_lo; p.order = a.order_q;
    static_assert(BM == kOrderTile, "the tile order is made for this tile size");
    p.S = a.S; p.Skv = a.Skv; p.off = a.off; p.Hq = a.Hq; p.Hkv = a.Hkv; p.G = a.Hq / a.Hkv;
    p.qmap = a.qmap; p.kvmap = a.kvmap;
    p.n_qtiles = (a.S + BM - 1) / BM;
    p.scale_log2 = a.scale * kLog2e;
    const dim3 grid = tile_rank_grid(a.Hq, a.B, p.n_qtiles), block(kThreads);
    hipLaunchKernelGGL((attn_fwd_kernel<D, VARLEN>), grid, block, 0, st, p);
    return launch_status();
}

}  // namespace

namespace sp {

sp_status launch_attn_fwd(const AttnArgs& a, hipStream_t st) {
    if ((int64_t)a.B * a.Hq > 0x7fffffff) return SP_ERR_SHAPE;
    const bool varlen = a.row_lo != nullptr;
    if (a.D == 128) return varlen ? launch<128, true>(a, st) : launch<128, false>(a, st);
    if (a.D == 64) return varlen ? launch<64, true>(a, st) : launch<64, false>(a, st);
    return SP_ERR_UNSUPPORTED;
}

}  // namespace sp
