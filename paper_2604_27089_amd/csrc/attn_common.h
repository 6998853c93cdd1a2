// Device-side building blocks shared by the attention kernels: vector types,
// the bf16 MFMA wrapper and its operand / accumulator lane layouts.
//
// v_mfma_f32_32x32x16_bf16 computes C[32x32] += A[32x16] * B[16x32] per wave.
// With lane l, lo = l % 32, hi = l / 32:
//   A operand: lane holds A[lo][8*hi + e], e = 0..7   (8 bf16 = 16 bytes)
//   B operand: lane holds B[8*hi + e][lo], e = 0..7
//   C/D      : lane holds C[8*(r/4) + 4*hi + r%4][lo] in register r = 0..15
// The contraction index only has to be paired consistently between A and B,
// which the kernels use to feed an accumulator straight back in as an operand:
// registers r = 8c .. 8c+7 of a C tile are rows {16c + 4*hi + e, 16c + 8 + 4*hi + e}.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace sp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// compile-time loop: f(std::integral_constant<int, I>{}) for I in [B, E)
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(static_cast<F&&>(f));
    }
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ u32x4 as_u32x4(bf16x8 v) { return __builtin_bit_cast(u32x4, v); }

// two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// registers [first, first+8) of an accumulator tile as a bf16 MFMA operand
__device__ __forceinline__ bf16x8 acc_to_operand(const f32x16& c, int first) {
    u32x4 r;
    r[0] = pack_bf16(c[first + 0], c[first + 1]);
    r[1] = pack_bf16(c[first + 2], c[first + 3]);
    r[2] = pack_bf16(c[first + 4], c[first + 5]);
    r[3] = pack_bf16(c[first + 6], c[first + 7]);
    return as_bf16x8(r);
}

// Position of a 4-row group inside its 16-row block in the "operand order" used
// for transposed LDS tiles: [0-3, 8-11, 4-7, 12-15], so that lane half `hi`
// reads its 8 contraction slots {4*hi + e, 8 + 4*hi + e} as one 16-byte load at
// offset 8*hi.
__device__ __forceinline__ int operand_pos4(int group4) {  // group4 = row/4
    const int blk = group4 >> 2, q4 = group4 & 3;
    const int pb = (q4 == 1) ? 2 : (q4 == 2) ? 1 : q4;
    return 16 * blk + 4 * pb;
}

// value held by the same lane of the other 32-lane half of the wave (v_permlane32_swap)
__device__ __forceinline__ float xhalf(float x) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    // swaps the upper half of the first operand with the lower half of the second
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    // r[0]: lanes 0-31 keep x, lanes 32-63 receive the lower half; r[1]: lanes 0-31 receive the upper half
    const uint32_t other = (__lane_id() < 32) ? r[1] : r[0];
    return __builtin_bit_cast(float, other);
}

// Transpose a 4 (rows) x 8 (cols) bf16 block held as four 16-byte row vectors
// into eight 8-byte column vectors (4 rows each).
__device__ __forceinline__ void transpose4x8(const u32x4 (&row)[4], u32x2 (&col)[8]) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        col[2 * w][0] = (row[0][w] & 0xffffu) | (row[1][w] << 16);
        col[2 * w][1] = (row[2][w] & 0xffffu) | (row[3][w] << 16);
        col[2 * w + 1][0] = (row[0][w] >> 16) | (row[1][w] & 0xffff0000u);
        col[2 * w + 1][1] = (row[2][w] >> 16) | (row[3][w] & 0xffff0000u);
    }
}

}  // namespace sp

// ---------------------------------------------------------------------------
// Unpadded, XOR-swizzled LDS tiles filled by direct global->LDS loads.
//
// A tile holds ROWS rows of D bf16 (D*2 bytes, CH = D/8 chunks of 16 bytes).
// Chunk c of row r is stored at chunk position c ^ swz<D>(r).  The swizzle is
// chosen so that both access patterns of the attention kernels are free of
// bank conflicts (64 banks x 4 bytes):
//   - row-major operand reads (ds_read_b128): 16 consecutive rows, same chunk;
//   - transposing reads (ds_read_b64_tr_b16): 4 consecutive rows (row % 4 = 0..3)
//     x 4 consecutive chunks per half-wave.
// ---------------------------------------------------------------------------
namespace sp {

template <int D>
__device__ __forceinline__ int swz(int row);
template <>
__device__ __forceinline__ int swz<128>(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
template <>
__device__ __forceinline__ int swz<64>(int row) { return (((row >> 1) & 1) << 2) | ((row >> 2) & 3); }

#define SP_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define SP_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// One wave copies 1024 contiguous LDS bytes: lane l supplies the 16 global bytes
// that land at lds_base + 16*l (lds_base must be wave-uniform).
__device__ __forceinline__ void dma16(const void* gsrc, void* lds_base) {
    __builtin_amdgcn_global_load_lds(SP_GPTR(gsrc), SP_LPTR(lds_base), 16, 0, 0);
}

// All of this wave's outstanding global loads (register and LDS destinations) have landed.
__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// Transposing LDS read: within each 16-lane block, lane i receives element i%4... see
// tile_dma_rows/tr_operand below for how the kernels use it.
__device__ __forceinline__ s16x4 lds_read_tr16(const void* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
}

// ---------------------------------------------------------------------------
// Hazard-proof build (-DSP_PADDED_MFMA): every assembly MFMA below is preceded by
// a full wait for outstanding LDS reads plus the two wait states a vector-ALU
// write needs before an MFMA reads it, and followed by the wait states after
// which any instruction may read its result; every partial LDS wait becomes a
// full one.  The arithmetic and its order are unchanged, so the padded build
// must give the regular build's bits: a test compares the two, which checks the
// hand-counted waits and instruction spacing of the regular build.
// ---------------------------------------------------------------------------
#ifdef SP_PADDED_MFMA
#define SP_MFMA_PRE "s_waitcnt lgkmcnt(0)\n\ts_nop 1\n\t"
#define SP_MFMA_POST "\n\ts_nop 15\n\ts_nop 7"
#define SP_LGKM(N) 0
#else
#define SP_MFMA_PRE ""
#define SP_MFMA_POST ""
#define SP_LGKM(N) (N)
#endif

// ---------------------------------------------------------------------------
// Asynchronous LDS operand reads with explicit waits.
//
// The compiler waits for ALL outstanding LDS reads before the first use of any
// of them; a software pipeline that keeps several operand reads in flight needs
// partial waits.  These helpers issue the read as opaque assembly (the compiler
// then tracks nothing) and lds_wait<N>(x) blocks until at most N younger LDS
// reads are outstanding, tying x to the wait so no use of x can be placed before
// it.  LDS reads of a wave complete in order, which makes the count exact.
// Rule: every value produced by lds_async_* must pass through lds_wait before
// it is used in any way, a register copy included: so such values never cross a
// control-flow join and are never packed into wider vectors before the wait.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)(p);
}
template <int OFF>
__device__ __forceinline__ u32x4 lds_async_b128(uint32_t addr) {
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
template <int OFF>
__device__ __forceinline__ u32x2 lds_async_tr16(uint32_t addr) {
    u32x2 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
template <int N>
__device__ __forceinline__ void lds_wait(u32x4& x) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(SP_LGKM(N)));
}
template <int N>
__device__ __forceinline__ void lds_wait(u32x2& x, u32x2& y) {
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(x), "+v"(y) : "n"(SP_LGKM(N)));
}

// ---------------------------------------------------------------------------
// Assembly MFMAs for the hand-scheduled backward kernels.
//
// In a kernel that may use more than 256 registers the compiler is free to put
// any MFMA accumulator into the accumulation registers, and does so even for
// tiles the vector ALU has to read and seed, paying a move per register each
// way; issued as assembly, the accumulator is constrained to the register file
// the kernel wants it in.  The compiler then no longer knows the instruction is
// an MFMA, so the caller owns the data hazards.  Those kernels run one wave per
// SIMD and are bound by how many instructions that lone wave can issue, so the
// helpers carry no padding in the regular build; the callers guarantee that
//   - no vector-ALU instruction writes an operand within the two instructions
//     before the MFMA (operands come from LDS reads, from earlier MFMAs, or from
//     arithmetic done at least one operand slot earlier);
//   - the vector ALU reads an MFMA's result only after enough later instructions
//     have issued to cover the 8-pass MFMA's result latency (in the kernels: two
//     independent MFMAs, or the vector-ALU chunk of an earlier step);
//   - back-to-back MFMAs on the same accumulator are interlocked by hardware.
// MFMAs ignore the EXEC mask: code that contains them must only be skipped by a
// truly scalar branch, so every wave-uniform condition guarding such code has
// to be built from scalar values (readfirstlane anything loaded per lane).
// Volatile assembly statements keep their order, which is what orders an MFMA
// after the wait that covers its operands.  W >= 0: that wait rides in the same
// statement.
//   mfma_v  : accumulator in vector registers       mfma_vc : ... starting from another tile
//   mfma_a  : accumulator in accumulation registers
//   *_ab    : the B operand lives in accumulation registers (resident operands)
// ---------------------------------------------------------------------------
template <int W>
__device__ __forceinline__ void mfma_v(f32x16& acc, const u32x4& a, const bf16x8& b) {
    if constexpr (W >= 0) asm volatile("s_waitcnt lgkmcnt(%3)\n\t" SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" SP_MFMA_POST : "+v"(acc) : "v"(a), "v"(b), "n"(W));
    else asm volatile(SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" SP_MFMA_POST : "+v"(acc) : "v"(a), "v"(b));
}
template <int W>
__device__ __forceinline__ void mfma_v(f32x16& acc, const u32x4& a, const u32x4& b) {
    if constexpr (W >= 0) asm volatile("s_waitcnt lgkmcnt(%3)\n\t" SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" SP_MFMA_POST : "+v"(acc) : "v"(a), "v"(b), "n"(W));
    else asm volatile(SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" SP_MFMA_POST : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_vc(f32x16& acc, const u32x4& a, const bf16x8& b, const f32x16& c) {
    asm volatile(SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" SP_MFMA_POST : "=&v"(acc) : "v"(a), "v"(b), "v"(c));
}
__device__ __forceinline__ void mfma_vc(f32x16& acc, const u32x4& a, const u32x4& b, const f32x16& c) {
    asm volatile(SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" SP_MFMA_POST : "=&v"(acc) : "v"(a), "v"(b), "v"(c));
}
__device__ __forceinline__ void mfma_a(f32x16& acc, const u32x4& a, const u32x4& b) {
    asm volatile(SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" SP_MFMA_POST : "+a"(acc) : "v"(a), "v"(b));
}
template <int W>
__device__ __forceinline__ void mfma_a_w(f32x16& acc, const u32x4& a, const u32x4& b) {
    if constexpr (W >= 0) asm volatile("s_waitcnt lgkmcnt(%3)\n\t" SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" SP_MFMA_POST : "+a"(acc) : "v"(a), "v"(b), "n"(W));
    else asm volatile(SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" SP_MFMA_POST : "+a"(acc) : "v"(a), "v"(b));
}
template <int W>
__device__ __forceinline__ void mfma_v_ab(f32x16& acc, const u32x4& a, const bf16x8& b) {
    if constexpr (W >= 0) asm volatile("s_waitcnt lgkmcnt(%3)\n\t" SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" SP_MFMA_POST : "+v"(acc) : "v"(a), "a"(b), "n"(W));
    else asm volatile(SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" SP_MFMA_POST : "+v"(acc) : "v"(a), "a"(b));
}
template <int W>
__device__ __forceinline__ void mfma_vc_ab(f32x16& acc, const u32x4& a, const bf16x8& b, const f32x16& c) {
    if constexpr (W >= 0) asm volatile("s_waitcnt lgkmcnt(%4)\n\t" SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" SP_MFMA_POST : "=&v"(acc) : "v"(a), "a"(b), "v"(c), "n"(W));
    else asm volatile(SP_MFMA_PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" SP_MFMA_POST : "=&v"(acc) : "v"(a), "a"(b), "v"(c));
}
// at most N of this wave's global loads (register and LDS destinations) are still in flight
template <int N>
__device__ __forceinline__ void vmem_wait() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
// Waits that tie the values they cover: used where the awaited registers are then combined into wider
// operands (the combination must not be scheduled before the wait).
template <int N>
__device__ __forceinline__ void lds_wait4(u32x4& a, u32x4& b, u32x4& c, u32x4& d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(SP_LGKM(N)));
}
template <int N>
__device__ __forceinline__ void lds_wait4(u32x2& a, u32x2& b, u32x2& c, u32x2& d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(SP_LGKM(N)));
}

// Per-lane description of the DMA loads that fill one ROWS x D tile with NW waves.
// (NW waves).  Instruction i (0 .. ROWS*CH/64-1) covers 64/CH rows; wave w issues i = w, w+NW, ...
// `wave` must be wave-uniform in the scalar sense (readfirstlane) so that LDS
// destinations are scalar.  Global addresses are a scalar tile base plus a 32-bit
// per-lane byte offset (rows of a tile span far less than 4 GiB).
template <int D, int ROWS, int NW = 4>
struct TileDma {
    static constexpr int CH = D / 8;
    static constexpr int RPI = 64 / CH;             // rows per instruction
    static constexpr int N_INSTR = ROWS * CH / 64;  // per tile, all waves
    static constexpr int PER_WAVE = N_INSTR / NW;
    static_assert(N_INSTR % NW == 0, "tile must split evenly over the waves");
    int row[PER_WAVE];          // row inside the tile this lane fetches for its k-th instruction
    uint32_t chunk_b[PER_WAVE]; // byte offset of the (swizzled) chunk this lane fetches inside that row
    uint32_t stride_b;          // global row stride in bytes
    __device__ __forceinline__ void init(int wave, int lane, size_t row_stride_elems) {
        stride_b = (uint32_t)(row_stride_elems * 2);
#pragma unroll
        for (int k = 0; k < PER_WAVE; ++k) {
            const int i = wave + NW * k;
            row[k] = RPI * i + lane / CH;
            chunk_b[k] = (uint32_t)(((lane % CH) ^ swz<D>(row[k])) * 16);
        }
    }
    // The K-th of this wave's PER_WAVE loads for the tile whose first row is at `tile` (a scalar
    // address); rows past the tile-relative row `lim` re-read row `lim` (their values are never used
    // unmasked).  Branch-free, so it can sit inside software-pipelined code.
    template <int K>
    __device__ __forceinline__ void issue_one(const __bf16* tile, int lim, __bf16* lds, int wave) const {
        const int r = row[K] < lim ? row[K] : lim;
        dma16(reinterpret_cast<const char*>(tile) + ((uint32_t)r * stride_b + chunk_b[K]), lds + (wave + NW * K) * 512);
    }
    __device__ __forceinline__ void issue(const __bf16* tile, int lim, __bf16* lds, int wave) const {
        static_for<0, PER_WAVE>([&](auto K) { issue_one<decltype(K)::value>(tile, lim, lds, wave); });
    }
};

// Byte offset, inside a swizzled tile, of the 16-byte row-major operand chunk (row, chunk).
template <int D>
__device__ __forceinline__ int tile_off_b128(int row, int chunk) {
    return row * (D * 2) + ((chunk ^ swz<D>(row)) * 16);
}

// Byte offset this lane passes to the transposing read so that, together with the other
// lanes of its 16-lane block, it receives rows {row0 .. row0+3} of column (col0 + i) where i
// is its index in the block: lane i supplies row row0 + i/4, columns col0 + 4*(i%4) .. +3.
template <int D>
__device__ __forceinline__ int tile_off_tr(int row0, int col0, int i16) {
    const int row = row0 + (i16 >> 2);
    const int col = col0 + 4 * (i16 & 3);
    return row * (D * 2) + (((col >> 3) ^ swz<D>(row)) * 16) + (col & 7) * 2;
}

}  // namespace sp
