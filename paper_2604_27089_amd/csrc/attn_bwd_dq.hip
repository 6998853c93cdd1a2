// dQ of causal grouped-query attention (paper Section 3.1: the rewritten graph
// must stay correct in the backward pass; Section 4.2 (breakdown analysis): the backward is where
// recomputation under activation checkpointing is paid).
//
//   dQ_i = scale * sum_{j<=i} dS_ij k_j,   dS_ij = P_ij (dO_i.v_j - Delta_i),
//   P_ij = exp(scale * q_i.k_j - LSE_i)
//
// As in the forward kernel, the general problem is S query rows against Skv
// keys with row i seeing keys j <= i + off (one step of a ring schedule,
// Section 4.1); the plain causal call is Skv = S, off = 0.
//
// One workgroup = 4 waves = 256 query rows of one query head, one wave per SIMD;
// a wave owns 64 rows (two 32-row blocks): their Q and dO stay resident as MFMA
// B operands (in accumulation registers), their dQ lives in accumulation
// registers that only MFMAs touch, and -LSE/scale and -Delta of the lane's row
// sit in register tiles that seed the S and dP accumulators through the MFMA C
// operand.  K/V stream through rings of eight 32-key LDS tiles (direct
// global->LDS loads issued six steps ahead, XOR-swizzled); every operand
// fetched from LDS feeds two MFMAs, one per row block.  Per 32-key step u:
//   S'^T = K.Q^T - LSE/scale, dP'^T = V.dO^T - Delta   (keys on the register axis,
//        one query per lane)
//   P = exp2(S' * scale*log2e), dS = P * dP'            (fp32 vector ALU, then bf16)
//   dQ^T += K^T.dS^T                                    (K^T from transposing LDS reads;
//        the dS^T accumulator tile is already a valid B operand)
//
// A lone wave issues in order, so the vector-ALU work is interleaved by hand
// into the MFMA stream.  One loop body runs three phases of D/16 operand slots
// (two MFMAs per slot):
//   S(u) + the loads of step u+6 | dP(u) + exponentials | dQ(u-1) + dS products
// i.e. the dQ contraction of a step is deferred into the next body.  The body is
// straight-line code: LDS operand reads are asynchronous, issued four slots
// ahead (across bodies) with one exact partial wait per pair of slots, and the
// body is instantiated once per ring position so that LDS addresses are
// immediates.
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int RPW = 64;           // query rows per wave
constexpr int BM = RPW * kWaves;  // query rows per workgroup
constexpr int BN = 32;            // keys per streamed tile = one step
constexpr int NBUF = 8;           // ring of streamed tiles (K and V each)
constexpr int LEAD = 6;           // a tile is loaded this many steps before its step

struct DqParams {
    const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* dO;
    const float* lse; const float* delta;
    __bf16* dq;
    const int32_t* row_lo;
    const int32_t* order;  // packed documents: query tiles in the order workgroups take them (or null)
    RowMap qmap, kvmap;
    int32_t S, Skv, off, Hq, Hkv, G, n_qtiles;  // S query rows, Skv keys; row i sees keys j <= i + off
    float scale, scale_log2;
};

template <int D, bool VARLEN>
__global__ __launch_bounds__(kThreads) void attn_bwd_dq_kernel(DqParams p) {
    constexpr int NS = D / 16;   // operand slots per phase (contraction steps over the head dim)
    constexpr int NDB = D / 32;  // 32-wide blocks of the head dim
    constexpr int TILE_B = BN * D * 2;
    constexpr int HALF_B = 16 * D * 2;  // 16 rows of a tile
    constexpr int KS = 0, VS = NBUF * TILE_B, SMEM = 2 * NBUF * TILE_B;
    static_assert(KS + (NBUF - 1) * TILE_B + HALF_B < 65536, "immediate LDS offsets must fit 16 bits");
    __shared__ __attribute__((aligned(1024))) char smem[SMEM];

    const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // heads vary fastest (they share K/V tiles), query tiles from the last (longest) to the first
    const int h = blockIdx.x % p.Hq, b = blockIdx.x / p.Hq;
    const int rank = (int)(blockIdx.y + kRankY * blockIdx.z);
    if (rank >= p.n_qtiles) return;  // the last z-slice of a grid of more than kRankY tiles may be ragged
    int qt = p.n_qtiles - 1 - rank;
    if (VARLEN && p.order) {  // longest tile first; clamped so that a bad entry cannot become a wild address
        const int v = __builtin_amdgcn_readfirstlane(p.order[rank]);
        qt = v < 0 ? 0 : (v < p.n_qtiles ? v : p.n_qtiles - 1);
    }
    const int g = h / p.G;
    const int S = p.S, Skv = p.Skv;
    const __bf16* qb_ = p.q + ((size_t)b * S * p.Hq + h) * D;
    const __bf16* dob = p.dO + ((size_t)b * S * p.Hq + h) * D;

    const int i0 = qt * BM;
    const int wrow0 = i0 + RPW * wave;  // first row of this wave

    // resident B operands (Q^T, dO^T columns of this lane's two rows) and accumulator seeds
    bf16x8 qreg[2][NS], doreg[2][NS];
    f32x16 seed_s[2], seed_p[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int row = wrow0 + 32 * qb + lo;
        const int rc = row < S ? row : S - 1;
#pragma unroll
        for (int kk = 0; kk < NS; ++kk) {
            qreg[qb][kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(qb_ + p.qmap.off(rc) + 16 * kk + 8 * hi));
            doreg[qb][kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(dob + p.qmap.off(rc) + 16 * kk + 8 * hi));
        }
        const float ls = -p.lse[((size_t)b * p.Hq + h) * S + rc] / p.scale;
        const float dl = -p.delta[((size_t)b * p.Hq + h) * S + rc];
#pragma unroll
        for (int r = 0; r < 16; ++r) { seed_s[qb][r] = ls; seed_p[qb][r] = dl; }
    }
    int wave_lo_max = 0, wg_lo_min = 0;
    int rlo_l[2] = {0, 0};  // packed documents: the first key this lane's rows may see (their document's start)
    if (VARLEN) {
        wave_lo_max = __builtin_amdgcn_readfirstlane(p.row_lo[(wrow0 + RPW - 1 < S ? wrow0 + RPW - 1 : S - 1)]);
        wg_lo_min = __builtin_amdgcn_readfirstlane(p.row_lo[i0]);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int row = wrow0 + 32 * qb + lo;
            rlo_l[qb] = p.row_lo[row < S ? row : S - 1];
        }
    }

    f32x16 dqacc[2][NDB];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) dqacc[qb][db][r] = 0.f;

    // LDS addresses of this lane's operand reads; everything that changes per step is an immediate
    const uint32_t sm = lds_addr(smem);
    uint32_t rk[NS], rv[NS];  // row-major operand (K, V rows): row lo, chunk 2*kk + hi
#pragma unroll
    for (int kk = 0; kk < NS; ++kk) {
        rk[kk] = sm + tile_off_b128<D>(lo, 2 * kk + hi);
        rv[kk] = rk[kk] + VS;
    }
    uint32_t tb[2][NDB];  // K^T operand: rows 8*half + 4*hi + (0..3) (+16 per 16-key half), cols 32*db + ...
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
            tb[half][db] = sm + tile_off_tr<D>(8 * half + 4 * hi, 32 * db + 16 * (lo >> 4), lo & 15);

    // the last key a row may see: i + off, at most the last key there is
    auto last_key = [&](int row) __attribute__((always_inline)) { return row + p.off < Skv - 1 ? row + p.off : Skv - 1; };
    const int jt_begin = VARLEN ? wg_lo_min / BN : 0;
    const int last_row = (i0 + BM - 1 < S ? i0 + BM - 1 : S - 1);
    const int jt_end = last_key(last_row) / BN + 1;  // exclusive
    const int total = jt_end - jt_begin;   // steps = key tiles, ascending

    // ---- global -> LDS loads of a step: K rows (PW), V rows (PW) per wave ----
    using Dma = TileDma<D, BN, kWaves>;
    constexpr int PW = Dma::PER_WAVE;
    constexpr int GROUP = 2 * PW;
    static_assert(GROUP <= NS, "one load per slot of the S phase");
    const uint32_t stride_b = p.kvmap.row_stride * 2;
    // byte offset, from the tile's first row, of the 16 bytes this lane fetches in its K-th load; rows past
    // `lim` (tile-relative) re-read row `lim` (they are never used unmasked)
    auto lane_off = [&](int K, int lim) __attribute__((always_inline)) {
        const int row = Dma::RPI * (wave + kWaves * K) + lane / Dma::CH;
        const uint32_t chunk_b = (uint32_t)(((lane % Dma::CH) ^ swz<D>(row)) * 16);
        return (uint32_t)(row < lim ? row : lim) * stride_b + chunk_b;
    };
    uint32_t voff[PW];  // offsets of the tile the load cursor is on
#pragma unroll
    for (int K = 0; K < PW; ++K) voff[K] = lane_off(K, BN - 1);
    const int jt_tail = (Skv % BN != 0) ? (Skv - 1) / BN : -1;  // the tile that runs past the last row, if any
    const int tiles_per_chunk_mask = (int)(p.kvmap.mask / BN);  // tiles per peer chunk - 1 (chunks are powers of two)

    // the step being loaded: scalar byte pointers to its tile in k and v
    struct LoadCursor { const char* k; const char* v; int jt, left; };
    LoadCursor dc;
    const size_t head0 = ((size_t)b * Skv * p.Hkv + g) * D * 2;
    const char* const k_head = reinterpret_cast<const char*>(p.k) + head0;
    const char* const v_head = reinterpret_cast<const char*>(p.v) + head0;
    const size_t tile_step_b = (size_t)BN * stride_b;
    // The tail tile is the last one the cursor can reach, and the cursor stays on it: its clamped lane offsets
    // replace the regular ones for good.
    auto enter_tile = [&]() __attribute__((always_inline)) {
        if (dc.jt == jt_tail) {  // rare
#pragma unroll
            for (int K = 0; K < PW; ++K) voff[K] = lane_off(K, Skv - 1 - dc.jt * BN);
        }
    };
    {
        dc.jt = jt_begin;
        const size_t off = p.kvmap.off(dc.jt * BN) * 2;
        dc.k = k_head + off;
        dc.v = v_head + off;
        dc.left = total - 1;
        enter_tile();
    }
    auto advance_load = [&]() __attribute__((always_inline)) {
        if (dc.left > 0) {  // past the last step the cursor stays (the padding steps re-read the last tile)
            --dc.left; dc.jt += 1;
            dc.k += tile_step_b; dc.v += tile_step_b;
            if ((dc.jt & tiles_per_chunk_mask) == 0) {  // rare: the first tile of the next peer's chunk
                const size_t off = p.kvmap.off(dc.jt * BN) * 2;
                dc.k = k_head + off; dc.v = v_head + off;
            }
            enter_tile();
        }
    };
    auto issue_load = [&](auto KC, int buf) __attribute__((always_inline)) {
        constexpr int K = decltype(KC)::value, KK = K % PW;
        const char* src = K < PW ? dc.k : dc.v;
        char* dst = smem + (K < PW ? KS : VS) + buf * TILE_B + (wave + kWaves * KK) * 1024;
        dma16(src + voff[KK], dst);
    };

    // ---- prologue: the first LEAD steps' tiles, and a finite stand-in for the deferred dQ of "step -1" ----
    int cur_jt = jt_begin;  // key tile of the step being computed
    int step_no = 0;        // its number (the step count is padded to a multiple of NBUF: steps >= total are not real)
    // steps whose S' needs masking: from the first whose keys reach past the last key the wave's first row
    // may see (and every padding step), and, for packed documents, those before the wave's last row's
    // document starts
    const int mask_from = (last_key(wrow0) / BN - jt_begin) < total ? (last_key(wrow0) / BN - jt_begin) : total;
    const int mask_until = VARLEN ? (wave_lo_max + BN - 1) / BN - jt_begin : 0;
    {
        static_for<0, PW>([&](auto K) { issue_load(K, NBUF - 1); });  // K rows of step 0 again, as the stand-in
        static_for<0, LEAD>([&](auto T) {
            static_for<0, GROUP>([&](auto K) { issue_load(K, decltype(T)::value); });
            advance_load();
        });
    }

    f32x16 sacc[2], pacc[2];
    u32x4 dsp[2][2][2];  // bf16 B operands [parity of the step][row block][16-key half]
#pragma unroll
    for (int par = 0; par < 2; ++par)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int c = 0; c < 2; ++c) dsp[par][qb][c] = u32x4{0, 0, 0, 0};

    // The operand slots of a body, x = 0 .. 3*NS-1 in the phases S | dP | dQ.  Reads of slot x are issued
    // kAhead slots early (behind the first MFMA of the issuing slot), possibly from the previous body (slots
    // x >= 3*NS name slots of the next body).  Waits happen once per pair of slots, at the even one.
    constexpr int P3 = 3 * NS;
    constexpr int kAhead = 4;
    auto nreads = [](int x) constexpr { return (x % P3) < 2 * NS ? 1 : 2; };
    // reads issued after those of slot s+1 by the time (even) slot s waits, which is before slot s issues
    // its own (none for the next body if `last`)
    auto young_reads = [=](int s, bool last) constexpr {
        int n = 0;
        for (int x = s + 2; x <= s - 1 + kAhead; ++x)
            if (!(last && x >= P3)) n += nreads(x);
        return n;
    };

    // in-flight operands (asynchronous reads: see the rule in attn_common.h)
    u32x4 ak[NS], av[NS];
    u32x2 t0[NS], t1[NS];

    // reads of slot s (0 .. 3*NS-1) of the body at ring position BUF
    auto issue_reads = [&](auto BUFC, auto SC) __attribute__((always_inline)) {
        constexpr int BUF = decltype(BUFC)::value, PBUF = (BUF + NBUF - 1) % NBUF, s = decltype(SC)::value;
        if constexpr (s < NS) {
            ak[s] = lds_async_b128<KS + BUF * TILE_B>(rk[s]);
        } else if constexpr (s < 2 * NS) {
            av[s - NS] = lds_async_b128<BUF * TILE_B>(rv[s - NS]);
        } else {
            constexpr int t = s - 2 * NS, c = t / NDB, db = t % NDB;
            t0[t] = lds_async_tr16<KS + PBUF * TILE_B + c * HALF_B>(tb[0][db]);
            t1[t] = lds_async_tr16<KS + PBUF * TILE_B + c * HALF_B>(tb[1][db]);
        }
    };

    // One body = step u at ring position BUF: (BUF-1)%8 holds step u-1 (its dQ is done here), (BUF+6)%8
    // receives step u+6.  FIRST: nothing was prefetched for this body (it follows the loop back-edge, which
    // asynchronous values must not cross); LAST: it prefetches nothing for the next body.  In the very
    // first body the deferred dQ multiplies the stand-in tile by zeros.
    auto body = [&](auto BUFC, auto FIRSTC, auto LASTC) __attribute__((always_inline)) {
        constexpr int BUF = decltype(BUFC)::value, DBUF = (BUF + LEAD) % NBUF, PAR = BUF % 2;
        constexpr bool FIRST = decltype(FIRSTC)::value, LAST = decltype(LASTC)::value;
        using NextBuf = std::integral_constant<int, (BUF + 1) % NBUF>;
        constexpr int EPM = 32 / (2 * NS);  // exponentials per MFMA in the dP phase
        constexpr int PPM = 16 / (2 * NS);  // dS pairs per MFMA in the dQ phase

        // exponentials of accumulator elements m*EPM .. of the step (element i = row block i/16, register
        // i%16); P stays in the S' registers
        auto exp_chunk = [&](auto MC) __attribute__((always_inline)) {
            constexpr int m = decltype(MC)::value;
            float t[EPM];
            static_for<0, EPM>([&](auto E) {
                constexpr int i = m * EPM + decltype(E)::value;
                t[decltype(E)::value] = sacc[i / 16][i % 16] * p.scale_log2;
            });
            static_for<0, EPM>([&](auto E) {
                constexpr int i = m * EPM + decltype(E)::value;
                sacc[i / 16][i % 16] = __builtin_amdgcn_exp2f(t[decltype(E)::value]);
            });
        };
        // dS of the pair j (0..15), for the dQ of the next body
        auto ds_pair = [&](auto JC) __attribute__((always_inline)) {
            constexpr int j = decltype(JC)::value, qb = j / 8, r = 2 * (j % 8);
            uint32_t w = pack_bf16(sacc[qb][r] * pacc[qb][r], sacc[qb][r + 1] * pacc[qb][r + 1]);
            asm volatile("" : "+v"(w));  // pins the arithmetic here: its only consumers are in the next body
            dsp[PAR][qb][r / 8][(r % 8) / 2] = w;
        };

        // Everybody is done with the previous body: nobody reads ring position (BUF+6)%8 = (BUF-2)%8 any
        // more.  This wave's loads of step u+1 have landed (those of the four steps after it may be in
        // flight); after the barrier so have everybody's.
        vmem_wait<(LEAD - 2) * GROUP>();
        __builtin_amdgcn_s_barrier();

        if constexpr (FIRST) static_for<0, kAhead>([&](auto XC) { issue_reads(BUFC, XC); });
        static_for<0, P3>([&](auto SC) {
            constexpr int s = decltype(SC)::value;
            constexpr bool even = s % 2 == 0;
            constexpr int W = even ? young_reads(s, LAST) : -1;  // reads allowed to stay in flight at the pair's wait
            __builtin_amdgcn_sched_barrier(0);
            // the reads this slot issues go out behind its first MFMA
            auto issue_slot = [&]() __attribute__((always_inline)) {
                constexpr int x = s + kAhead;
                if constexpr (x < P3) issue_reads(BUFC, std::integral_constant<int, x>{});
                else if constexpr (!LAST) issue_reads(NextBuf{}, std::integral_constant<int, x - P3>{});
                __builtin_amdgcn_sched_barrier(0);
            };
            if constexpr (s < NS) {
                // ---- S(u); the loads of step u+6 ----
                if constexpr (s == 0) mfma_vc_ab<W>(sacc[0], ak[s], qreg[0][s], seed_s[0]);
                else mfma_v_ab<W>(sacc[0], ak[s], qreg[0][s]);
                __builtin_amdgcn_sched_barrier(0);
                issue_slot();
                if constexpr (s < GROUP) issue_load(SC, DBUF);
                // the cursor moves on in the first slot without a load (scalar work between the slot's read and
                // its second MFMA, where the compiler would otherwise put a wait state)
                if constexpr (s == GROUP) advance_load();
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (s == 0) mfma_vc_ab<-1>(sacc[1], ak[s], qreg[1][s], seed_s[1]);
                else mfma_v_ab<-1>(sacc[1], ak[s], qreg[1][s]);
            } else if constexpr (s < 2 * NS) {
                // ---- dP(u), exponentials ----
                // Exponential chunk m runs behind MFMA m+1 of the phase (the last one behind the first MFMA
                // of the dQ phase): two MFMAs have then issued since the last write of S', which covers the
                // wait states between an MFMA and a vector-ALU read of its result.
                constexpr int kk = s - NS;
                if constexpr (kk == 0) mfma_vc_ab<W>(pacc[0], av[kk], doreg[0][kk], seed_p[0]);
                else mfma_v_ab<W>(pacc[0], av[kk], doreg[0][kk]);
                __builtin_amdgcn_sched_barrier(0);
                issue_slot();
                if constexpr (kk > 0) exp_chunk(std::integral_constant<int, 2 * kk - 1>{});
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (kk == 0) mfma_vc_ab<-1>(pacc[1], av[kk], doreg[1][kk], seed_p[1]);
                else mfma_v_ab<-1>(pacc[1], av[kk], doreg[1][kk]);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (kk == 0) {
                    // Causal / document mask: hidden positions get S' = -inf, i.e. P = 0.  Index by index only
                    // on steps that reach the diagonal (or are padding) and, with packed documents, on the
                    // step in which some row's document starts.  A row whose document starts after the step's
                    // keys sees none of them: all 16 of its S' take one select on a per-lane flag (a select, not
                    // arithmetic: S' of such a pair may be anything, a NaN included).  A wave whose rows
                    // straddle a document boundary is in that state for every step of the earlier document;
                    // masked index by index, it held the whole workgroup back on its longest walk.
                    bool elementwise = step_no >= mask_from;
                    if (VARLEN && step_no < mask_until) {  // some row's document starts at or after this step's keys
                        const int j0 = cur_jt * BN;
                        const bool dead0 = rlo_l[0] >= j0 + BN, dead1 = rlo_l[1] >= j0 + BN;
                        elementwise = elementwise ||
                                      __builtin_amdgcn_ballot_w64((rlo_l[0] > j0 && rlo_l[0] < j0 + BN) ||
                                                                  (rlo_l[1] > j0 && rlo_l[1] < j0 + BN)) != 0;
                        if (!elementwise && __builtin_amdgcn_ballot_w64(dead0 || dead1) != 0) {
                            asm volatile("" ::: "memory");  // keeps this a branch
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                sacc[0][r] = dead0 ? -__builtin_inff() : sacc[0][r];
                                sacc[1][r] = dead1 ? -__builtin_inff() : sacc[1][r];
                            }
                        }
                    }
                    if (elementwise) {  // rare
                        asm volatile("" ::: "memory");  // keeps this a branch (not selects executed on every step)
                        const int j0 = cur_jt * BN;
                        const bool real = step_no < total;
#pragma unroll
                        for (int qb = 0; qb < 2; ++qb) {
                            const int row = wrow0 + 32 * qb + (int)(__lane_id() & 31);
                            const int rlo = VARLEN ? rlo_l[qb] : 0;  // first key the row may see
                            const int rhi = row + p.off < p.Skv - 1 ? row + p.off : p.Skv - 1;  // and the last
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int key = j0 + 8 * (r / 4) + 4 * (int)(__lane_id() >> 5) + (r % 4);
                                const bool vis = real && key <= rhi && key >= rlo;
                                sacc[qb][r] = vis ? sacc[qb][r] : -__builtin_inff();
                            }
                        }
                    }
                }
                exp_chunk(std::integral_constant<int, 2 * kk>{});
            } else {
                // ---- dQ(u-1), dS products of step u (pair chunk m behind MFMA m+1, as above) ----
                constexpr int t = s - 2 * NS, c = t / NDB, db = t % NDB;
                const u32x4 kt = {t0[t][0], t0[t][1], t1[t][0], t1[t][1]};
                mfma_a_w<W>(dqacc[0][db], kt, dsp[1 - PAR][0][c]);
                __builtin_amdgcn_sched_barrier(0);
                issue_slot();
                if constexpr (t == 0) exp_chunk(std::integral_constant<int, 2 * NS - 1>{});
                else static_for<0, PPM>([&](auto J) { ds_pair(std::integral_constant<int, (2 * t - 1) * PPM + decltype(J)::value>{}); });
                __builtin_amdgcn_sched_barrier(0);
                mfma_a(dqacc[1][db], kt, dsp[1 - PAR][1][c]);
                __builtin_amdgcn_sched_barrier(0);
                static_for<0, PPM>([&](auto J) { ds_pair(std::integral_constant<int, (2 * t) * PPM + decltype(J)::value>{}); });
                if constexpr (t == NS - 1) static_for<0, PPM>([&](auto J) { ds_pair(std::integral_constant<int, (2 * t + 1) * PPM + decltype(J)::value>{}); });
            }
        });
        __builtin_amdgcn_sched_barrier(0);
        ++step_no;
        if (step_no < total) cur_jt += 1;
        if constexpr (GROUP >= NS) advance_load();
    };

    // Eight steps per iteration, one per ring position; the step count is rounded up to a multiple of
    // eight with steps whose P is all zero (they re-read the last tile).
    for (int u = 0; u < total; u += NBUF) {
        body(std::integral_constant<int, 0>{}, std::true_type{}, std::false_type{});
        body(std::integral_constant<int, 1>{}, std::false_type{}, std::false_type{});
        body(std::integral_constant<int, 2>{}, std::false_type{}, std::false_type{});
        body(std::integral_constant<int, 3>{}, std::false_type{}, std::false_type{});
        body(std::integral_constant<int, 4>{}, std::false_type{}, std::false_type{});
        body(std::integral_constant<int, 5>{}, std::false_type{}, std::false_type{});
        body(std::integral_constant<int, 6>{}, std::false_type{}, std::false_type{});
        body(std::integral_constant<int, 7>{}, std::false_type{}, std::true_type{});
    }

    // ---- the deferred dQ of the last step (ring position 7, dS of parity 1) ----
    {
        static_for<0, NS>([&](auto TC) {
            constexpr int t = decltype(TC)::value, c = t / NDB, db = t % NDB;
            u32x2 h0 = lds_async_tr16<KS + (NBUF - 1) * TILE_B + c * HALF_B>(tb[0][db]);
            u32x2 h1 = lds_async_tr16<KS + (NBUF - 1) * TILE_B + c * HALF_B>(tb[1][db]);
            lds_wait<0>(h0, h1);
            const u32x4 kt = {h0[0], h0[1], h1[0], h1[1]};
            dqacc[0][db] = mfma32(as_bf16x8(kt), as_bf16x8(dsp[1][0][c]), dqacc[0][db]);
            dqacc[1][db] = mfma32(as_bf16x8(kt), as_bf16x8(dsp[1][1][c]), dqacc[1][db]);
        });
    }
    wait_vmem();  // no direct-to-LDS load may outlive the workgroup's LDS allocation

    // ---- write dQ (scaled): accumulator rows = d, column = this lane's query ----
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int row = wrow0 + 32 * qb + lo;
        if (row < S) {
            __bf16* out = p.dq + ((size_t)b * S * p.Hq + h) * D + p.qmap.off(row);
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
    p.lse = a.lse; p.delta = a.delta; p.dq = (__bf16*)a.dq; p.row_lo = a.row_lo; p.order = a.order_q;
    static_assert(BM == kOrderTile, "the tile order is made for this tile size");
    p.S = a.S; p.Skv = a.Skv; p.off = a.off; p.Hq = a.Hq; p.Hkv = a.Hkv; p.G = a.Hq / a.Hkv;
    p.qmap = a.qmap; p.kvmap = a.kvmap;
    p.n_qtiles = (a.S + BM - 1) / BM;
    p.scale = a.scale; p.scale_log2 = a.scale * kLog2e;
    const dim3 grid = tile_rank_grid(a.Hq, a.B, p.n_qtiles);
    hipLaunchKernelGGL((attn_bwd_dq_kernel<D, VARLEN>), grid, dim3(kThreads), 0, st, p);
    return launch_status();
}

}  // namespace

namespace sp {

sp_status launch_attn_bwd_dq(const AttnArgs& a, hipStream_t st) {
    if ((int64_t)a.B * a.Hq > 0x7fffffff) return SP_ERR_SHAPE;
    const bool varlen = a.row_lo != nullptr;
    if (a.D == 128) return varlen ? launch<128, true>(a, st) : launch<128, false>(a, st);
    if (a.D == 64) return varlen ? launch<64, true>(a, st) : launch<64, false>(a, st);
    return SP_ERR_UNSUPPORTED;
}

}  // namespace sp
