// dK and dV of causal grouped-query attention (paper Section 3.1: the rewritten
// graph must stay correct in the backward pass; Section 4.2 (breakdown analysis): the backward is
// where recomputation under activation checkpointing is paid).
//
//   dV_j = sum_{a in group} sum_{i>=j} P_ij dO_i
//   dK_j = scale * sum_{a in group} sum_{i>=j} dS_ij q_i,   dS_ij = P_ij (dO_i.v_j - Delta_i)
//
// One workgroup = 4 waves = 256 keys of one KV head, one wave per SIMD; a wave
// owns 64 keys (two 32-key blocks): their K stays in registers as MFMA B operand,
// their V sits in LDS for the whole kernel, and their dK, dV live in 256
// accumulation registers that only MFMAs touch.  A streamed operand fetched from
// LDS feeds two MFMAs (one per key block).
//
// The Q/dO rows of the G query heads of the group stream through a ring of four
// 32-row LDS tiles (direct global->LDS loads issued two steps ahead,
// XOR-swizzled), from the last row down to the diagonal so that co-resident
// workgroups read the same rows at the same time.  Per 32-row step u and wave:
//   S' = Q.K^T - LSE/scale, dP' = dO.V^T - Delta   (the subtractions ride in the
//        accumulator initial value, fetched per row from LDS; masked positions
//        start from -inf instead)
//   P = exp2(S' * scale*log2e), dS = P * dP'       (fp32 vector ALU, then bf16)
//   dV += P^T.dO, dK += dS^T.Q                     (P and dS accumulator tiles are
//        already valid A operands; dO^T and Q^T come from transposing LDS reads)
//
// A lone wave issues in order, so the vector-ALU work is interleaved by hand
// into the MFMA stream.  One loop body runs four phases of D/16 operand slots
// (two MFMAs per slot):
//   S(u) | dK(u-1) + first half of exp | dP(u) + second half of exp | dV(u) + dS products
// i.e. the dK contraction of a step is deferred into the next body, where it
// and the dP contraction give the exponentials of the new step something to
// hide behind.  The body is straight-line code: every LDS operand read is
// asynchronous, issued two slots ahead with exact partial waits, the tile loads
// of step u+2 are spread over the S phase, and the body is instantiated once per
// ring position so that all LDS addresses are immediates.
#include "attn_common.h"
#include "sp_common.h"

namespace {

using namespace sp;

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int KPW = 64;            // keys per wave
constexpr int BNK = KPW * kWaves;  // keys per workgroup
constexpr int BMQ = 32;            // query rows per streamed tile = one step
constexpr int NBUF = 4;            // ring of streamed tiles

struct DkdvParams {
    const __bf16* q; const __bf16* k; const __bf16* v; const __bf16* dO;
    const float* aux;  // per 32-row tile: 32 x -LSE/scale then 32 x -Delta; [B*Hq, S_pad/32, 2, 32]
    __bf16* dk; __bf16* dv;
    float* part;  // nsplit > 1: fp32 partial sums, [2 (dK unscaled, dV)][nsplit][B, Skv, Hkv, D]
    const int32_t* row_hi;
    const int32_t* order;  // packed documents: key tiles in the order workgroups take them (or null)
    RowMap qmap, kvmap;
    int32_t B, batch_fastest;
    int32_t S, Skv, off, S_pad, Hq, Hkv, G, n_ktiles, nsplit;  // S query rows, Skv keys; row i sees keys j <= i + off
    float scale, scale_log2;
};

// 16 accumulator registers from the four 16-byte per-row reads of one lane
__device__ __forceinline__ void seeds_to_acc(f32x16& acc, const u32x4 (&s)[4]) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const uint32_t u = s[r / 4][r % 4];  // (through a scalar: bit-casting a vector element expression directly is not reliable)
        acc[r] = __uint_as_float(u);
    }
}

template <int D, bool VARLEN, bool SPLIT>
__global__ __launch_bounds__(kThreads) void attn_bwd_dkdv_kernel(DkdvParams p) {
    constexpr int NS = D / 16;   // operand slots per phase (contraction steps over the head dim)
    constexpr int NDB = D / 32;  // 32-wide blocks of the head dim
    constexpr int TILE_B = BMQ * D * 2;
    constexpr int HALF_B = 16 * D * 2;  // 16 rows of a tile
    constexpr int QS = 0, DOS = NBUF * TILE_B, VS = 2 * NBUF * TILE_B, VW_B = KPW * D * 2;
    constexpr int AUX = VS + kWaves * VW_B, AUX_SLOT = 1024, AUX_W = NBUF * AUX_SLOT;
    constexpr int SMEM = AUX + kWaves * AUX_W;
    static_assert(DOS + (NBUF - 1) * TILE_B + HALF_B < 65536, "immediate LDS offsets must fit 16 bits");
    __shared__ __attribute__((aligned(1024))) char smem[SMEM];

    const int tid = threadIdx.x, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // earliest key tiles (most rows to visit) first; the nsplit workgroups that share a key tile are neighbours
    const int nsplit = SPLIT ? p.nsplit : 1;
    // Grid: (key tile x chunk, KV head, batch entry) for a single sequence; with several sequences the batch
    // entry and KV head vary fastest instead, (KV head + Hkv * batch entry, key tile x chunk), so that every
    // sequence's longest key tiles are dispatched before anybody's short ones (sequence by sequence, the last
    // sequence's longest tile started when the grid was two thirds done: 16 x 4096 rows 710 -> 510 us).
    const int chunk_id = p.batch_fastest ? blockIdx.y : blockIdx.x;
    int jt = SPLIT ? chunk_id / nsplit : chunk_id;
    const int split = SPLIT ? chunk_id % nsplit : 0;
    if (VARLEN && p.order) {  // longest tile first; clamped so that a bad entry cannot become a wild address
        const int v = __builtin_amdgcn_readfirstlane(p.order[jt]);
        jt = v < 0 ? 0 : (v < p.n_ktiles ? v : p.n_ktiles - 1);
    }
    const int g = p.batch_fastest ? blockIdx.x % p.Hkv : blockIdx.y;
    const int b = p.batch_fastest ? blockIdx.x / p.Hkv : blockIdx.z;
    const int S = p.S, Skv = p.Skv;
    const __bf16* kb = p.k + ((size_t)b * Skv * p.Hkv + g) * D;
    const __bf16* vb = p.v + ((size_t)b * Skv * p.Hkv + g) * D;

    const int j0 = jt * BNK;
    const int wkey0 = j0 + KPW * wave;  // first key of this wave

    // resident B operand: K^T columns of this lane's two keys
    bf16x8 kreg[2][NS];
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk) {
        const int key = wkey0 + 32 * kbk + lo;
        const int key_c = key < Skv ? key : Skv - 1;
#pragma unroll
        for (int kk = 0; kk < NS; ++kk) {
            kreg[kbk][kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(kb + p.kvmap.off(key_c) + 16 * kk + 8 * hi));
        }
    }
    int wave_hi_min = S, wg_hi_max = S;
    int khi_l[2] = {S, S};  // packed documents: one past the last row that may see this lane's keys (their document's end)
    if (VARLEN) {
        wave_hi_min = __builtin_amdgcn_readfirstlane(p.row_hi[(wkey0 < S ? wkey0 : S - 1)]);
        wg_hi_max = __builtin_amdgcn_readfirstlane(p.row_hi[(j0 + BNK - 1 < S ? j0 + BNK - 1 : S - 1)]);
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk) {
            const int key = wkey0 + 32 * kbk + lo;
            khi_l[kbk] = p.row_hi[key < S ? key : S - 1];
        }
    }

    f32x16 dkacc[2][NDB], dvacc[2][NDB];
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) { dkacc[kbk][db][r] = 0.f; dvacc[kbk][db][r] = 0.f; }

    // LDS addresses of this lane's operand reads; everything that changes per step is an immediate
    const uint32_t sm = lds_addr(smem);
    uint32_t rb[NS];  // row-major operand (Q, dO rows): row lo, chunk 2*kk + hi
    uint32_t vr[NS];  // the same chunk of this wave's V rows
#pragma unroll
    for (int kk = 0; kk < NS; ++kk) {
        rb[kk] = sm + tile_off_b128<D>(lo, 2 * kk + hi);
        vr[kk] = rb[kk] + VS + wave * VW_B;
    }
    uint32_t tb[2][NDB];  // transposed operand (Q^T, dO^T): rows 8*half + 4*hi + (0..3) (+16 per 16-row step), cols 32*db + ...
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
            tb[half][db] = sm + tile_off_tr<D>(8 * half + 4 * hi, 32 * db + 16 * (lo >> 4), lo & 15);
    const uint32_t ab = sm + AUX + wave * AUX_W + 16 * hi;  // per-row scalars: rows 8*g4 + 4*hi .. +3

    const int it_begin = (j0 > p.off ? j0 - p.off : 0) / BMQ;  // tile holding the first row that sees the first key
    const int it_end = (wg_hi_max + BMQ - 1) / BMQ;  // exclusive
    const int n_it = it_end - it_begin;
    // Steps are (head in group, row tile) pairs, heads ascending, rows descending inside a head.  The
    // key tile's step sequence is cut into nsplit contiguous chunks, one per workgroup; a chunk may be
    // empty (its workgroup then contributes zeros).
    const int total_all = n_it * p.G;
    const int per_split = (total_all + nsplit - 1) / nsplit;
    int s_begin = split * per_split < total_all ? split * per_split : total_all;
    const int s_end = s_begin + per_split < total_all ? s_begin + per_split : total_all;
    const int total = s_end - s_begin;
    if (total == 0) s_begin = 0;  // keeps the prologue's loads on valid addresses
    const int head_first = s_begin / n_it;             // first head (inside the group) of this chunk
    const int it_first = it_end - 1 - s_begin % n_it;  // and its first row tile

    // ---- global -> LDS loads of a step: per-row scalars (1), Q rows (PW), dO rows (PW) per wave ----
    using Dma = TileDma<D, BMQ, kWaves>;
    constexpr int PW = Dma::PER_WAVE;
    constexpr int GROUP = 1 + 2 * PW;
    static_assert(GROUP <= NS, "one load per slot of the S phase");
    const uint32_t stride_b = p.qmap.row_stride * 2;
    // byte offset, from the tile's first row, of the 16 bytes this lane fetches in its K-th load; rows past
    // `lim` (tile-relative) re-read row `lim` (they are never used unmasked)
    auto lane_off = [&](int K, int lim) __attribute__((always_inline)) {
        const int row = Dma::RPI * (wave + kWaves * K) + lane / Dma::CH;
        const uint32_t chunk_b = (uint32_t)(((lane % Dma::CH) ^ swz<D>(row)) * 16);
        return (uint32_t)(row < lim ? row : lim) * stride_b + chunk_b;
    };
    uint32_t voff[PW];
#pragma unroll
    for (int K = 0; K < PW; ++K) voff[K] = lane_off(K, BMQ - 1);
    const uint32_t aux_lane_b = 16 * (lane & 15);  // 256 bytes per tile; lanes 16.. duplicate, their LDS bytes are padding
    const int it_tail = (S % BMQ != 0) ? (S - 1) / BMQ : -1;  // the tile that runs past the last row, if any

    // the step being loaded: scalar byte pointers to its tile in q, dO and the per-row scalars
    struct LoadCursor { const char* q; const char* dO; const char* aux; int it, left; };
    LoadCursor dc;
    // byte offsets of the current head (inside the batch entry) in q/dO and of the current tile's rows
    size_t q_head_b = ((size_t)b * S * p.Hq + (size_t)g * p.G + head_first) * D * 2;
    {
        dc.it = it_first;
        const size_t off = p.qmap.off(dc.it * BMQ) * 2;
        dc.q = reinterpret_cast<const char*>(p.q) + q_head_b + off;
        dc.dO = reinterpret_cast<const char*>(p.dO) + q_head_b + off;
        dc.aux = reinterpret_cast<const char*>(p.aux) + (((size_t)b * p.Hq + (size_t)g * p.G + head_first) * (p.S_pad / 32) + dc.it) * 256;
        dc.left = total - 1;
    }
    const size_t aux_jump_b = ((size_t)(p.S_pad / 32) + (size_t)(n_it - 1)) * 256;
    auto advance_load = [&]() __attribute__((always_inline)) {
        if (dc.left > 0) {  // past the last step the cursor stays (the padding steps re-read the last tile)
            --dc.left;
            if (dc.it == it_begin) {  // first tile of a head -> last tile of the next
                dc.it = it_end - 1; q_head_b += (size_t)D * 2; dc.aux += aux_jump_b;
            } else {
                dc.it -= 1; dc.aux -= 256;
            }
            const size_t off = q_head_b + p.qmap.off(dc.it * BMQ) * 2;
            dc.q = reinterpret_cast<const char*>(p.q) + off;
            dc.dO = reinterpret_cast<const char*>(p.dO) + off;
        }
    };
    auto issue_load = [&](auto KC, int buf) __attribute__((always_inline)) {
        constexpr int K = decltype(KC)::value;
        if constexpr (K == 0) {
            dma16(dc.aux + aux_lane_b, smem + AUX + wave * AUX_W + buf * AUX_SLOT);
        } else {
            constexpr int KK = (K - 1) % PW;
            uint32_t off = voff[KK];
            if (dc.it == it_tail) off = lane_off(KK, S - 1 - dc.it * BMQ);  // rare
            const char* src = K <= PW ? dc.q : dc.dO;
            char* dst = smem + (K <= PW ? QS : DOS) + buf * TILE_B + (wave + kWaves * KK) * 1024;
            dma16(src + off, dst);
        }
    };

    // ---- prologue: V (resident), a finite stand-in tile for the deferred dK of "step -1", steps 0 and 1 ----
    int cur_it = it_first;    // row tile of the step being computed
    int step_no = 0;          // its number (the step count is padded to a multiple of four: steps >= total are not real)
    // row tiles whose S' needs masking: those holding a row that does not see the wave's last key, and those
    // reaching the end of the first key's document (dense: the end of the sequence)
    const int last_hidden = wkey0 + KPW - 2 - p.off;  // last row that does not see all the wave's keys
    const int it_mask_lo = last_hidden >= 0 ? last_hidden / BMQ : -1;
    const int it_mask_hi = (wave_hi_min - 31 + BMQ - 1) / BMQ;
    {
        TileDma<D, BNK, kWaves> vdma;
        vdma.init(wave, lane, p.kvmap.row_stride);
        vdma.issue(vb + p.kvmap.off(j0), Skv - 1 - j0, reinterpret_cast<__bf16*>(smem + VS), wave);
        static_for<1, PW + 1>([&](auto K) { issue_load(K, 3); });  // Q rows of step 0 again, as the stand-in
        static_for<0, GROUP>([&](auto K) { issue_load(K, 0); });
        advance_load();
        static_for<0, GROUP>([&](auto K) { issue_load(K, 1); });
        advance_load();
        vmem_wait<GROUP>();  // everything but the loads of step 1 has landed (this wave's share) ...
        __builtin_amdgcn_s_barrier();  // ... and everybody else's
    }

    f32x16 sacc[2], pacc[2];
    u32x4 pp[2][2], dsp[2][2];  // bf16 A operands [key block][16-row half]: P of the step, dS of the previous step
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int c = 0; c < 2; ++c) { dsp[kbk][c] = u32x4{0, 0, 0, 0}; pp[kbk][c] = u32x4{0, 0, 0, 0}; }

    // The operand slots of a body, x = 0 .. 4*NS-1 in the phases S | dK | dP | dV.  Reads of slot x are issued
    // ahead(x) slots early, possibly from the previous body (slots x >= 4*NS name slots of the next body).
    // Waits happen once per pair of slots, at the even one.
    constexpr int P4 = 4 * NS;
    auto nreads = [](int x) constexpr {  // LDS reads of slot x (first S and dP slots: plus the four per-row reads)
        const int s = x % P4;
        return s == 0 ? 5 : s < NS ? 1 : s < 2 * NS ? 2 : s == 2 * NS ? 7 : s < 3 * NS ? 3 : 2;
    };
    auto ahead = [](int x) constexpr {
        const int s = x % P4;
        return (s >= 2 * NS && s < 3 * NS) ? 3 : 4;
    };
    constexpr int kMaxAhead = 4;
    // reads issued after those of slot s+1 by the time (even) slot s waits, which is before slot s issues
    // its own (none for the next body if `last`)
    auto young_reads = [=](int s, bool last) constexpr {
        int n = 0;
        for (int x = s + 2; x <= s + kMaxAhead; ++x)
            if (x - ahead(x) <= s - 1 && !(last && x >= P4)) n += nreads(x);
        return n;
    };

    // in-flight operands (asynchronous reads: see the rule in attn_common.h)
    u32x4 aq[NS], ad[NS], bv0[NS], bv1[NS], sds[4], sdp[4];
    u32x2 bq0[NS], bq1[NS], bd0[NS], bd1[NS];

    // reads of slot s (0 .. 4*NS-1) of the body at ring position BUF
    auto issue_reads = [&](auto BUFC, auto SC) __attribute__((always_inline)) {
        constexpr int BUF = decltype(BUFC)::value, PBUF = (BUF + 3) % NBUF, s = decltype(SC)::value;
        if constexpr (s < NS) {
            if constexpr (s == 0) static_for<0, 4>([&](auto G4) { sds[G4] = lds_async_b128<BUF * AUX_SLOT + 32 * decltype(G4)::value>(ab); });
            aq[s] = lds_async_b128<QS + BUF * TILE_B>(rb[s]);
        } else if constexpr (s < 2 * NS) {
            constexpr int t = s - NS, c = t / NDB, db = t % NDB;
            bq0[t] = lds_async_tr16<QS + PBUF * TILE_B + c * HALF_B>(tb[0][db]);
            bq1[t] = lds_async_tr16<QS + PBUF * TILE_B + c * HALF_B>(tb[1][db]);
        } else if constexpr (s < 3 * NS) {
            constexpr int kk = s - 2 * NS;
            if constexpr (kk == 0) static_for<0, 4>([&](auto G4) { sdp[G4] = lds_async_b128<BUF * AUX_SLOT + 128 + 32 * decltype(G4)::value>(ab); });
            ad[kk] = lds_async_b128<DOS + BUF * TILE_B>(rb[kk]);
            bv0[kk] = lds_async_b128<0>(vr[kk]);
            bv1[kk] = lds_async_b128<32 * D * 2>(vr[kk]);
        } else {
            constexpr int t = s - 3 * NS, c = t / NDB, db = t % NDB;
            bd0[t] = lds_async_tr16<DOS + BUF * TILE_B + c * HALF_B>(tb[0][db]);
            bd1[t] = lds_async_tr16<DOS + BUF * TILE_B + c * HALF_B>(tb[1][db]);
        }
    };

    // One body = step u at ring position BUF: (BUF+3)%4 holds step u-1 (its dK is done here), (BUF+1)%4 step
    // u+1, (BUF+2)%4 receives step u+2.  FIRST: nothing was prefetched for this body (it follows the loop
    // back-edge, which asynchronous values must not cross); LAST: it prefetches nothing for the next body.
    // In the very first body the deferred dK multiplies zeros by the stand-in tile.
    auto body = [&](auto BUFC, auto FIRSTC, auto LASTC) __attribute__((always_inline)) {
        constexpr int BUF = decltype(BUFC)::value, DBUF = (BUF + 2) % NBUF;
        constexpr bool FIRST = decltype(FIRSTC)::value, LAST = decltype(LASTC)::value;
        using NextBuf = std::integral_constant<int, (BUF + 1) % NBUF>;
        constexpr int EPM = 32 / (4 * NS);  // exponentials per MFMA in the dK and dP phases (32 MFMAs, 32 elements)
        constexpr int PPM = 16 / (2 * NS);  // dS pairs per MFMA in the dV phase

        // Vector-ALU work of MFMA position m (0 .. 4*NS-1) of the dK and dP phases: the exponentials of
        // accumulator elements m*EPM .. (element i = key block i/16, register i%16; P stays in the S'
        // registers), and the bf16 packing of the pairs completed by the previous position (so that no
        // pack directly follows the exponential it reads).
        auto pack_pair = [&](auto JC) __attribute__((always_inline)) {
            constexpr int j = decltype(JC)::value, kbk = j / 8, r = 2 * (j % 8);
            pp[kbk][r / 8][(r % 8) / 2] = pack_bf16(sacc[kbk][r], sacc[kbk][r + 1]);
        };
        auto exp_chunk = [&](auto MC) __attribute__((always_inline)) {
            constexpr int m = decltype(MC)::value;
            float t[EPM];
            static_for<0, EPM>([&](auto E) {
                constexpr int i = m * EPM + decltype(E)::value;
                t[decltype(E)::value] = sacc[i / 16][i % 16] * p.scale_log2;
            });
            if constexpr (m > 0) static_for<((m - 1) * EPM) / 2, (m * EPM) / 2>([&](auto J) { pack_pair(J); });
            static_for<0, EPM>([&](auto E) {
                constexpr int i = m * EPM + decltype(E)::value;
                sacc[i / 16][i % 16] = __builtin_amdgcn_exp2f(t[decltype(E)::value]);
            });
        };
        // dS of the pair j (0..15)
        auto ds_pair = [&](auto JC) __attribute__((always_inline)) {
            constexpr int j = decltype(JC)::value, kbk = j / 8, r = 2 * (j % 8);
            uint32_t w = pack_bf16(sacc[kbk][r] * pacc[kbk][r], sacc[kbk][r + 1] * pacc[kbk][r + 1]);
            asm volatile("" : "+v"(w));  // pins the arithmetic here: its only consumers are in the next body
            dsp[kbk][r / 8][(r % 8) / 2] = w;
        };

        if constexpr (FIRST) {
            static_for<0, kMaxAhead>([&](auto XC) {
                if constexpr (decltype(XC)::value - ahead(decltype(XC)::value) < 0) issue_reads(BUFC, XC);
            });
        }
        static_for<0, P4>([&](auto SC) {
            constexpr int s = decltype(SC)::value;
            constexpr bool even = s % 2 == 0;
            constexpr int W = even ? young_reads(s, LAST) : -1;  // reads allowed to stay in flight at the pair's wait
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (s == 2 * NS) {
                // Everybody is past the dK phase: nobody reads ring position (BUF+3)%4 any more.  This wave's
                // loads of step u+1 have landed (those of step u+2, issued in this body, may be in flight);
                // after the barrier so have everybody's.
                vmem_wait<GROUP>();
                __builtin_amdgcn_s_barrier();
            }
            // the reads this slot issues go out behind its first MFMA (a read holds the wave's issue for
            // about half an MFMA; in front of the MFMA that time would be lost)
            auto issue_slot = [&]() __attribute__((always_inline)) {
                static_for<1, kMaxAhead + 1>([&](auto AC) {
                    constexpr int x = s + decltype(AC)::value;
                    if constexpr (x - ahead(x) == s) {
                        if constexpr (x < P4) issue_reads(BUFC, std::integral_constant<int, x>{});
                        else if constexpr (!LAST) issue_reads(NextBuf{}, std::integral_constant<int, x - P4>{});
                    }
                });
                __builtin_amdgcn_sched_barrier(0);
            };
            if constexpr (s < NS) {
                // ---- S(u); the loads of step u+2 ----
                if constexpr (s == 0) {
                    lds_wait4<W>(sds[0], sds[1], sds[2], sds[3]);
                    f32x16 seed;
                    seeds_to_acc(seed, sds);
                    mfma_vc(sacc[0], aq[s], kreg[0][s], seed);
                    __builtin_amdgcn_sched_barrier(0);
                    issue_slot();
                    issue_load(std::integral_constant<int, 0>{}, DBUF);
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_vc(sacc[1], aq[s], kreg[1][s], seed);
                } else {
                    mfma_v<W>(sacc[0], aq[s], kreg[0][s]);
                    __builtin_amdgcn_sched_barrier(0);
                    issue_slot();
                    if constexpr (s < GROUP) issue_load(std::integral_constant<int, s>{}, DBUF);
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_v<-1>(sacc[1], aq[s], kreg[1][s]);
                }
            } else if constexpr (s < 2 * NS) {
                // ---- dK(u-1), exponentials of key block 0 ----
                // Exponential chunk m runs behind MFMA m+1 of the dK and dP phases taken together (the last
                // one behind the first MFMA of the dV phase): two MFMAs have then issued since the last write
                // of S', which covers the wait states between an MFMA and a vector-ALU read of its result.
                constexpr int t = s - NS, c = t / NDB, db = t % NDB;
                const u32x4 bqt = {bq0[t][0], bq0[t][1], bq1[t][0], bq1[t][1]};
                mfma_a_w<W>(dkacc[0][db], dsp[0][c], bqt);
                __builtin_amdgcn_sched_barrier(0);
                issue_slot();
                if constexpr (t > 0) exp_chunk(std::integral_constant<int, 2 * t - 1>{});
                __builtin_amdgcn_sched_barrier(0);
                mfma_a(dkacc[1][db], dsp[1][c], bqt);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (t == 0) {
                    // Causal / document mask: hidden positions get S' = -inf, i.e. P = 0.  Index by index only
                    // on row tiles that reach the diagonal, on padding steps and, with packed documents, on the
                    // row tile in which some key's document ends.  A key whose document ends before the row
                    // tile is seen by none of its rows: all 16 of its S' take one select on a per-lane flag
                    // (a select, not arithmetic: S' of such a pair may be anything, a NaN included).  A wave
                    // whose keys straddle a document boundary is in that state for every row tile of the later
                    // document; masked index by index, it held the whole workgroup back on its longest walk.
                    bool elementwise = cur_it <= it_mask_lo || step_no >= total;
                    if (VARLEN && cur_it >= it_mask_hi) {  // rows at or past the end of the first key's document
                        const int q0 = cur_it * BMQ;
                        const bool dead0 = khi_l[0] <= q0, dead1 = khi_l[1] <= q0;
                        elementwise = elementwise ||
                                      __builtin_amdgcn_ballot_w64((khi_l[0] > q0 && khi_l[0] < q0 + BMQ) ||
                                                                  (khi_l[1] > q0 && khi_l[1] < q0 + BMQ)) != 0;
                        if (!elementwise && __builtin_amdgcn_ballot_w64(dead0 || dead1) != 0) {
                            asm volatile("" ::: "memory");  // keeps this a branch
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                sacc[0][r] = dead0 ? -__builtin_inff() : sacc[0][r];
                                sacc[1][r] = dead1 ? -__builtin_inff() : sacc[1][r];
                            }
                        }
                    }
                    if (!VARLEN && cur_it >= it_mask_hi) elementwise = true;  // rows past the end of the sequence
                    if (elementwise) {  // rare
                        asm volatile("" ::: "memory");  // keeps this a branch (not selects executed on every step)
                        const int q0 = cur_it * BMQ;
                        const bool real = step_no < total;
#pragma unroll
                        for (int kbk = 0; kbk < 2; ++kbk) {
                            const int key = wkey0 + 32 * kbk + (int)(__lane_id() & 31);
                            const int key_hi = VARLEN ? khi_l[kbk] : S;  // one past the last row that may see the key
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int row = q0 + 8 * (r / 4) + 4 * (int)(__lane_id() >> 5) + (r % 4);
                                const bool vis = real && row + p.off >= key && row < key_hi;
                                sacc[kbk][r] = vis ? sacc[kbk][r] : -__builtin_inff();
                            }
                        }
                    }
                }
                exp_chunk(std::integral_constant<int, 2 * t>{});
            } else if constexpr (s < 3 * NS) {
                // ---- dP(u), exponentials of key block 1 ----
                constexpr int kk = s - 2 * NS;
                if constexpr (kk == 0) {
                    lds_wait4<W>(sdp[0], sdp[1], sdp[2], sdp[3]);
                    f32x16 seed;
                    seeds_to_acc(seed, sdp);
                    mfma_vc(pacc[0], ad[kk], bv0[kk], seed);
                    __builtin_amdgcn_sched_barrier(0);
                    issue_slot();
                    exp_chunk(std::integral_constant<int, 2 * (NS + kk) - 1>{});
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_vc(pacc[1], ad[kk], bv1[kk], seed);
                } else {
                    mfma_v<W>(pacc[0], ad[kk], bv0[kk]);
                    __builtin_amdgcn_sched_barrier(0);
                    issue_slot();
                    exp_chunk(std::integral_constant<int, 2 * (NS + kk) - 1>{});
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_v<-1>(pacc[1], ad[kk], bv1[kk]);
                }
                __builtin_amdgcn_sched_barrier(0);
                exp_chunk(std::integral_constant<int, 2 * (NS + kk)>{});
            } else {
                // ---- dV(u), dS products (pair chunk m behind MFMA m+1 of the phase, as above) ----
                constexpr int t = s - 3 * NS, c = t / NDB, db = t % NDB;
                const u32x4 bdo = {bd0[t][0], bd0[t][1], bd1[t][0], bd1[t][1]};
                mfma_a_w<W>(dvacc[0][db], pp[0][c], bdo);
                __builtin_amdgcn_sched_barrier(0);
                issue_slot();
                if constexpr (t == 0) {
                    exp_chunk(std::integral_constant<int, 4 * NS - 1>{});
                    static_for<((4 * NS - 1) * EPM) / 2, 16>([&](auto J) { pack_pair(J); });  // the last pair(s) of P
                } else {
                    static_for<0, PPM>([&](auto J) { ds_pair(std::integral_constant<int, (2 * t - 1) * PPM + decltype(J)::value>{}); });
                }
                __builtin_amdgcn_sched_barrier(0);
                mfma_a(dvacc[1][db], pp[1][c], bdo);
                __builtin_amdgcn_sched_barrier(0);
                static_for<0, PPM>([&](auto J) { ds_pair(std::integral_constant<int, (2 * t) * PPM + decltype(J)::value>{}); });
                if constexpr (t == NS - 1) static_for<0, PPM>([&](auto J) { ds_pair(std::integral_constant<int, (2 * t + 1) * PPM + decltype(J)::value>{}); });
            }
        });
        __builtin_amdgcn_sched_barrier(0);
        ++step_no;
        if (step_no < total) cur_it = (cur_it == it_begin) ? it_end - 1 : cur_it - 1;
        advance_load();
    };

    // Four steps per iteration, one per ring position; the step count is rounded up to a multiple of four
    // with steps whose P is all zero (they re-read the last tile).
    for (int u = 0; u < total; u += NBUF) {
        body(std::integral_constant<int, 0>{}, std::true_type{}, std::false_type{});
        body(std::integral_constant<int, 1>{}, std::false_type{}, std::false_type{});
        body(std::integral_constant<int, 2>{}, std::false_type{}, std::false_type{});
        body(std::integral_constant<int, 3>{}, std::false_type{}, std::true_type{});
    }

    // ---- the deferred dK of the last step ----
    {
        constexpr uint32_t qoff = QS + (NBUF - 1) * TILE_B;
        static_for<0, NS>([&](auto TC) {
            constexpr int t = decltype(TC)::value, c = t / NDB, db = t % NDB;
            u32x2 h0 = lds_async_tr16<c * HALF_B>(tb[0][db] + qoff);
            u32x2 h1 = lds_async_tr16<c * HALF_B>(tb[1][db] + qoff);
            lds_wait<0>(h0, h1);
            const u32x4 bqt = {h0[0], h0[1], h1[0], h1[1]};
            dkacc[0][db] = mfma32(as_bf16x8(dsp[0][c]), as_bf16x8(bqt), dkacc[0][db]);
            dkacc[1][db] = mfma32(as_bf16x8(dsp[1][c]), as_bf16x8(bqt), dkacc[1][db]);
        });
    }
    wait_vmem();  // no direct-to-LDS load may outlive the workgroup's LDS allocation

    // ---- write dK and dV: accumulator rows = keys, column = d ----
    if constexpr (SPLIT) {
        // fp32 partial sums of this chunk (dK unscaled); the reduction kernel adds the chunks in a fixed order
        const size_t n_out = (size_t)p.B * Skv * p.Hkv * D;
        float* pk = p.part + (size_t)split * n_out;
        float* pv = pk + (size_t)nsplit * n_out;
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int krow = wkey0 + 32 * kbk + 8 * (r / 4) + 4 * hi + (r % 4);
                    if (krow < Skv) {
                        const size_t off = (((size_t)b * Skv + krow) * p.Hkv + g) * D + 32 * db + lo;
                        pk[off] = dkacc[kbk][db][r];
                        pv[off] = dvacc[kbk][db][r];
                    }
                }
    } else {
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int krow = wkey0 + 32 * kbk + 8 * (r / 4) + 4 * hi + (r % 4);
                    if (krow < Skv) {
                        const size_t off = ((size_t)b * Skv * p.Hkv + g) * D + p.kvmap.off(krow) + 32 * db + lo;
                        p.dk[off] = (__bf16)(dkacc[kbk][db][r] * p.scale);
                        p.dv[off] = (__bf16)dvacc[kbk][db][r];
                    }
                }
    }
}

// dK = scale * sum of the chunks' partial sums, dV = sum of theirs; four elements per thread.  The
// partial sums are dense [B, S, Hkv*D]; the outputs follow `map`.
__global__ __launch_bounds__(256) void dkdv_reduce_kernel(const float* __restrict__ part, __bf16* __restrict__ dk,
                                                         __bf16* __restrict__ dv, int64_t n_out, int32_t nsplit,
                                                         float scale, RowMap map, int32_t S, int32_t HD) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n_out) return;  // n_out is a multiple of 4 (D is)
    const int64_t br = i / HD;  // b*S + row
    const int64_t bb = br / S;
    const size_t o = (size_t)bb * S * HD + map.off((int32_t)(br - bb * S)) + (size_t)(i - br * HD);
    f32x4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
    for (int32_t s = 0; s < nsplit; ++s) {
        sk += *reinterpret_cast<const f32x4*>(part + (size_t)s * n_out + i);
        sv += *reinterpret_cast<const f32x4*>(part + ((size_t)nsplit + s) * n_out + i);
    }
    u32x2 wk, wv;
    wk[0] = pack_bf16(sk[0] * scale, sk[1] * scale); wk[1] = pack_bf16(sk[2] * scale, sk[3] * scale);
    wv[0] = pack_bf16(sv[0], sv[1]); wv[1] = pack_bf16(sv[2], sv[3]);
    *reinterpret_cast<u32x2*>(dk + o) = wk;
    *reinterpret_cast<u32x2*>(dv + o) = wv;
}

template <int D, bool VARLEN>
sp_status launch(const AttnArgs& a, hipStream_t st) {
    DkdvParams p;
    p.q = (const __bf16*)a.q; p.k = (const __bf16*)a.k; p.v = (const __bf16*)a.v; p.dO = (const __bf16*)a.dO;
    p.aux = a.aux; p.dk = (__bf16*)a.dk; p.dv = (__bf16*)a.dv; p.row_hi = a.row_hi; p.order = a.order_k;
    static_assert(BNK == kOrderTile, "the tile order is made for this tile size");
    p.S = a.S; p.Skv = a.Skv; p.off = a.off; p.S_pad = a.S_pad; p.Hq = a.Hq; p.Hkv = a.Hkv; p.G = a.Hq / a.Hkv;
    p.qmap = a.qmap; p.kvmap = a.kvmap;
    p.n_ktiles = (a.Skv + BNK - 1) / BNK;
    p.nsplit = a.dkdv_splits; p.part = a.dkdv_part;
    p.scale = a.scale; p.scale_log2 = a.scale * kLog2e;
    if (p.nsplit < 1 || (p.nsplit > 1 && !p.part)) return SP_ERR_WORKSPACE;
    p.B = a.B;
    p.batch_fastest = a.B > 1 && (int64_t)p.n_ktiles * p.nsplit <= 65535 && (int64_t)a.Hkv * a.B <= 0x7fffffff;
    dim3 grid(p.n_ktiles * p.nsplit, a.Hkv, a.B);
    if (p.batch_fastest) grid = dim3(a.Hkv * a.B, p.n_ktiles * p.nsplit, 1);
    if (p.nsplit > 1) hipLaunchKernelGGL((attn_bwd_dkdv_kernel<D, VARLEN, true>), grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL((attn_bwd_dkdv_kernel<D, VARLEN, false>), grid, dim3(kThreads), 0, st, p);
    if (launch_status() != SP_OK) return SP_ERR_LAUNCH;
    if (p.nsplit > 1) {
        const int64_t n_out = (int64_t)a.B * a.Skv * a.Hkv * D;
        const int64_t blocks = (n_out / 4 + 255) / 256;
        hipLaunchKernelGGL(dkdv_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p.part, p.dk, p.dv, n_out,
                           p.nsplit, p.scale, a.kvmap, a.Skv, a.Hkv * D);
    }
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
