// Sequence<->head re-layout around the all-to-all (paper Section 2, Figure 1:
// the exchange toggles activations between [S/P, all heads] and
// [S, heads/P]; Section 3.1 challenge 1: its buffers are sized by batch,
// sequence and model dimension).
//
// pack   (to_head):  out[b, p*S_l + s, j, :] = in[b, s, p*h + j, :]
// unpack (to_seq) :  out[b, s, p*h + j, :]   = in[b, p*S_l + s, j, :]
//
// Both are permutations of runs of h*D*elem_bytes contiguous bytes, moved as
// 16-byte vectors.  The kernel walks the OUTPUT linearly (fully coalesced
// stores) and gathers; a gather run is at least 256 bytes long for every
// workload shape, so reads are coalesced too.  HBM-bound: one read and one
// write of every byte, no reuse, hence non-temporal accesses.
#include "sp_common.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kUnroll = 8;  // 16-byte vectors in flight per thread

// n_vec   : total 16-byte vectors
// run     : vectors per contiguous run (h * D * elem_bytes / 16)
// S_l, P  : tokens per rank, ranks
// TO_HEAD : pack if true, unpack otherwise
// IDX     : uint32_t when every vector index fits 32 bits (cheap divisions)
template <bool TO_HEAD, typename IDX>
__global__ __launch_bounds__(kThreads) void relayout_kernel(const u32x4* __restrict__ in,
                                                           u32x4* __restrict__ out,
                                                           uint64_t n_vec, uint32_t run,
                                                           uint32_t S_l, uint32_t P) {
    const IDX base = (IDX)blockIdx.x * (IDX)(kThreads * kUnroll) + (IDX)threadIdx.x;
    u32x4 val[kUnroll];
    IDX dst[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const IDX o = base + (IDX)(u * kThreads);
        dst[u] = o;
        if (o < (IDX)n_vec) {
            // output run index -> (b, outer, inner); input run index swaps outer/inner
            const IDX orun = o / (IDX)run;
            const IDX r = o - orun * (IDX)run;
            IDX irun;
            if (TO_HEAD) {  // out runs ordered (b, p, s); in runs ordered (b, s, p)
                const IDX bp = orun / (IDX)S_l;
                const IDX s = orun - bp * (IDX)S_l;
                const IDX b = bp / (IDX)P;
                const IDX p = bp - b * (IDX)P;
                irun = (b * (IDX)S_l + s) * (IDX)P + p;
            } else {        // out runs ordered (b, s, p); in runs ordered (b, p, s)
                const IDX bs = orun / (IDX)P;
                const IDX p = orun - bs * (IDX)P;
                const IDX b = bs / (IDX)S_l;
                const IDX s = bs - b * (IDX)S_l;
                irun = (b * (IDX)P + p) * (IDX)S_l + s;
            }
            val[u] = __builtin_nontemporal_load(in + (size_t)(irun * (IDX)run + r));
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
        if (dst[u] < (IDX)n_vec) __builtin_nontemporal_store(val[u], out + (size_t)dst[u]);
}

// Fast path for power-of-two runs (every workload shape): no divisions by the run.  One workgroup moves
// kFastThreads*UNROLL consecutive vectors of one (batch, peer) slab of the head-side tensor, which is
// contiguous there; on the sequence side the same vectors are S_l runs strided by P*run.
// grid.x = peer + P * chunk, grid.y = batch: the PEER varies fastest, so that the workgroups in flight
// together touch whole rows of the sequence-side tensor (P adjacent runs) instead of one run out of
// every P.  With the chunk fastest, a slab's reads land on one out of every P address granules at a time
// and leave most memory channels idle in turn: 6.0 TB/s against 6.5 on the 70B-shaped Q shard, where a
// plain linear copy of the same bytes reaches 6.5.  Block and unroll sizes come from a sweep on MI355X
// with cold buffers: one 16-byte vector per thread and 512 threads; more vectors in flight per thread lose
// 4 % (two) to 9 % (four).
constexpr int kFastThreads = 512;
constexpr int kFastUnroll = 1;
template <bool TO_HEAD, int UNROLL>
__global__ __launch_bounds__(kFastThreads) void relayout_pow2_kernel(const u32x4* __restrict__ in,
                                                                u32x4* __restrict__ out, uint32_t slab_vec,
                                                                uint32_t log2_run, uint32_t S_l, uint32_t P) {
    const uint32_t chunk = blockIdx.x / P, p = blockIdx.x - chunk * P, b = blockIdx.y;
    const uint32_t run_mask = (1u << log2_run) - 1u;
    const size_t batch_vec = (size_t)slab_vec * P;  // vectors per batch element
    const u32x4* src = in + (size_t)b * batch_vec;
    u32x4* dst = out + (size_t)b * batch_vec;
    const uint32_t head_base = p * slab_vec;        // slab p of the head-side tensor
    const uint32_t e0 = chunk * (kFastThreads * UNROLL) + threadIdx.x;
    u32x4 val[UNROLL];
    uint32_t to[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const uint32_t e = e0 + u * kFastThreads;        // vector inside the slab
        const uint32_t s = e >> log2_run, r = e & run_mask;
        const uint32_t seq_idx = ((s * P + p) << log2_run) + r;
        const uint32_t head_idx = head_base + e;
        to[u] = TO_HEAD ? head_idx : seq_idx;
        if (e < slab_vec) val[u] = __builtin_nontemporal_load(src + (TO_HEAD ? seq_idx : head_idx));
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
        if (e0 + u * kFastThreads < slab_vec) __builtin_nontemporal_store(val[u], dst + to[u]);
}

// Unpack with linear stores: one workgroup writes kFastThreads*UNROLL consecutive vectors of the
// sequence-side tensor and gathers them from the P slabs of the head-side tensor (runs and P powers of
// two): both sides of the copy then advance through whole rows.  Used for runs of 2 KB and more (6.3 TB/s
// on the 70B-shaped Q shard); on shorter runs the slab-wise kernel above is as fast.
// grid = (ceil(P*S_l*run / (kFastThreads*UNROLL)), B).
template <int UNROLL>
__global__ __launch_bounds__(kFastThreads) void unpack_pow2_linear_store_kernel(const u32x4* __restrict__ in,
                                                                           u32x4* __restrict__ out,
                                                                           uint32_t slab_vec, uint32_t log2_run,
                                                                           uint32_t log2_P) {
    const uint32_t b = blockIdx.y;
    const uint32_t batch_vec = slab_vec << log2_P;
    const u32x4* src = in + (size_t)b * batch_vec;
    u32x4* dst = out + (size_t)b * batch_vec;
    const uint32_t run_mask = (1u << log2_run) - 1u, p_mask = (1u << log2_P) - 1u;
    const uint32_t o0 = blockIdx.x * (kFastThreads * UNROLL) + threadIdx.x;
    u32x4 val[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const uint32_t o = o0 + u * kFastThreads;  // vector of the sequence-side tensor: (s, p, r)
        const uint32_t r = o & run_mask, sp_ = o >> log2_run, p = sp_ & p_mask, s = sp_ >> log2_P;
        if (o < batch_vec) val[u] = __builtin_nontemporal_load(src + (size_t)(p * slab_vec + (s << log2_run) + r));
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
        if (o0 + u * kFastThreads < batch_vec) __builtin_nontemporal_store(val[u], dst + (o0 + u * kFastThreads));
}

}  // namespace

namespace sp {

sp_status launch_relayout(const void* in, void* out, int64_t B, int64_t S_l, int64_t H, int64_t D,
                          int32_t P, int32_t elem_bytes, bool to_head, hipStream_t st) {
    const uint64_t h = (uint64_t)(H / P);
    const uint64_t run = h * (uint64_t)D * (uint64_t)elem_bytes / 16;
    const uint64_t n_vec = (uint64_t)B * (uint64_t)S_l * (uint64_t)P * run;
    const uint64_t per_block = (uint64_t)kThreads * kUnroll;
    const uint64_t blocks = (n_vec + per_block - 1) / per_block;
    if (blocks == 0) return SP_OK;
    if (blocks > 0x7fffffffull || run > 0xffffffffull) return SP_ERR_SHAPE;
    if ((uint64_t)S_l > 0xffffffffull) return SP_ERR_SHAPE;
    const uint64_t slab = (uint64_t)S_l * run;  // vectors of one (batch, peer) slab
    if ((run & (run - 1)) == 0 && slab * (uint64_t)P + 4096 < 0xffffffffull && P <= 65535 && B <= 65535) {
        uint32_t lr = 0;
        while ((1ull << lr) < run) ++lr;
        const uint64_t pb = (uint64_t)kFastThreads * kFastUnroll;
        if (!to_head && (P & (P - 1)) == 0 && run >= 128) {  // measured: linear stores win from 2 KB runs on
            uint32_t lp = 0;
            while ((1 << lp) < P) ++lp;
            dim3 g3((unsigned)((slab * (uint64_t)P + pb - 1) / pb), (unsigned)B);
            hipLaunchKernelGGL((unpack_pow2_linear_store_kernel<kFastUnroll>), g3, dim3(kFastThreads), 0, st,
                               (const u32x4*)in, (u32x4*)out, (uint32_t)slab, lr, lp);
            return launch_status();
        }
        const uint64_t chunks = (slab + pb - 1) / pb;
        if (chunks * (uint64_t)P <= 0x7fffffffull) {
            dim3 g2((unsigned)(chunks * (uint64_t)P), (unsigned)B);
#define SP_FAST(TH, U)                                                                                   \
    hipLaunchKernelGGL((relayout_pow2_kernel<TH, U>), g2, dim3(kFastThreads), 0, st, (const u32x4*)in,    \
                       (u32x4*)out, (uint32_t)slab, lr, (uint32_t)S_l, (uint32_t)P)
            if (to_head) SP_FAST(true, kFastUnroll); else SP_FAST(false, kFastUnroll);
#undef SP_FAST
            return launch_status();
        }
    }
    dim3 grid((unsigned)blocks), block(kThreads);
    const bool small = n_vec + per_block < 0xffffffffull;  // every index, tail included, fits u32
#define SP_RELAYOUT(TH, IDX)                                                                     \
    hipLaunchKernelGGL((relayout_kernel<TH, IDX>), grid, block, 0, st, (const u32x4*)in,          \
                       (u32x4*)out, n_vec, (uint32_t)run, (uint32_t)S_l, (uint32_t)P)
    if (to_head) { if (small) SP_RELAYOUT(true, uint32_t); else SP_RELAYOUT(true, uint64_t); }
    else         { if (small) SP_RELAYOUT(false, uint32_t); else SP_RELAYOUT(false, uint64_t); }
#undef SP_RELAYOUT
    return launch_status();
}

}  // namespace sp
