// Pointwise operators between the matrix multiplications of a Llama layer, on
// one device's [S/P, model dim] token shard: RMS normalisation, rotary position
// embedding and the SwiGLU gate, forward and backward.  The paper's
// activation-checkpointing strategy has every operator outside the attention
// layer rematerialised in the backward pass (Section 3.2), so each of these
// runs twice per training step; the models it evaluates are Llama models
// (Section 4 setup).  Outside attention a device holds part of the sequence with
// the full model dimension (Section 2, Figure 1).
//
// All of them stream: every element is read once and written once, in 16-byte
// vectors with non-temporal accesses; arithmetic is fp32, results are rounded
// to bf16 once.  HBM-bound.
#include "sp_common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ void widen(const u32x4& v, float (&f)[8]) {
    const bf16x8 b = __builtin_bit_cast(bf16x8, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (float)b[e];
}
__device__ __forceinline__ u32x4 narrow(const float (&f)[8]) {
    u32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const f32x2 p = {f[2 * e], f[2 * e + 1]};
        r[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
    }
    return r;
}
__device__ __forceinline__ u32x4 ld16(const void* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); }
__device__ __forceinline__ void st16(void* p, const u32x4& v) { __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p)); }
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// ------------------------------------------------------------------ RMS norm, forward
// One wave per row; the row stays in registers between the sum of squares and the scaling.
// Lane l owns the 8-column vectors number l, l+64, ... (NV of them, C <= 512*NV).
template <int NV>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const __bf16* __restrict__ x, const __bf16* __restrict__ w,
                                                         __bf16* __restrict__ y, float* __restrict__ rstd,
                                                         int64_t T, int32_t C, float eps) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= T) return;
    const __bf16* xr = x + row * C;
    // loads are unconditional (columns past the row's end re-read its last vector and count as zeros), so
    // that all of a lane's loads are in flight together
    u32x4 xv[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c0 = (j * 64 + lane) * 8;
        xv[j] = ld16(xr + (c0 < C ? c0 : C - 8));
    }
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c0 = (j * 64 + lane) * 8;
        float f[8];
        widen(xv[j], f);
        float s8 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s8 += f[e] * f[e];
        ss += c0 < C ? s8 : 0.f;
    }
    ss = wave_sum(ss);
    const float r = 1.0f / sqrtf(ss / (float)C + eps);
    if (lane == 0) rstd[row] = r;
    __bf16* yr = y + row * C;
    u32x4 wv[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c0 = (j * 64 + lane) * 8;
        wv[j] = *reinterpret_cast<const u32x4*>(w + (c0 < C ? c0 : C - 8));
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c0 = (j * 64 + lane) * 8;
        float f[8], g[8];
        widen(xv[j], f);
        widen(wv[j], g);
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = f[e] * r * g[e];
        if (c0 < C) st16(yr + c0, narrow(f));
    }
}

// ------------------------------------------------------------------ RMS norm, backward
//   g = dy * w,  dx = g * rstd - x * rstd^3 * (sum_c g x) / C,  dw = sum_t dy * x * rstd
// One workgroup per row, rows dealt round-robin to a fixed number of workgroups; thread t owns the 8-column
// vectors number t, t+256, ... (NVT of them, C <= 2048*NVT) and keeps their dw terms in registers over all its
// rows, so a workgroup's partial row of dw needs no reduction; the row's sum_c g x goes wave sums -> LDS ->
// every thread adds the four.  rmsnorm_dw_kernel adds the partial rows in a fixed order.
template <int NVT>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const __bf16* __restrict__ x, const __bf16* __restrict__ w,
                                                         const float* __restrict__ rstd, const __bf16* __restrict__ dy,
                                                         __bf16* __restrict__ dx, float* __restrict__ part,
                                                         int64_t T, int32_t C) {
    __shared__ float wsum[2][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float dwacc[NVT][8];
    u32x4 wv[NVT];  // w of the thread's columns (zeros past the row's end, which also zeroes every term there)
#pragma unroll
    for (int j = 0; j < NVT; ++j) {
        const int c0 = (j * 256 + (int)threadIdx.x) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) dwacc[j][e] = 0.f;
        wv[j] = *reinterpret_cast<const u32x4*>(w + (c0 < C ? c0 : C - 8));
        if (c0 >= C) wv[j] = u32x4{0, 0, 0, 0};
    }
    // The next row's x and dy are requested before this row's sum goes through the barrier, so a
    // workgroup always has two rows of loads in flight (one row at a time left the memory system idle
    // during every reduction: 4.5 TB/s).
    auto fetch = [&](int64_t row, u32x4 (&xn)[NVT], u32x4 (&dn)[NVT]) __attribute__((always_inline)) {
        const __bf16* xr = x + row * C;
        const __bf16* dyr = dy + row * C;
#pragma unroll
        for (int j = 0; j < NVT; ++j) {
            const int c0 = (j * 256 + (int)threadIdx.x) * 8;
            const int cc = c0 < C ? c0 : C - 8;
            xn[j] = ld16(xr + cc);
            dn[j] = ld16(dyr + cc);
        }
    };
    u32x4 xv[NVT], dv[NVT], xn[NVT], dn[NVT];
    if ((int64_t)blockIdx.x < T) fetch(blockIdx.x, xn, dn);
    int par = 0;
    for (int64_t row = blockIdx.x; row < T; row += gridDim.x, par ^= 1) {
#pragma unroll
        for (int j = 0; j < NVT; ++j) { xv[j] = xn[j]; dv[j] = dn[j]; }
        if (row + gridDim.x < T) fetch(row + gridDim.x, xn, dn);
        const float r = rstd[row];
        float dot = 0.f;
#pragma unroll
        for (int j = 0; j < NVT; ++j) {
            float xf[8], df[8], wf[8];
            widen(xv[j], xf);
            widen(dv[j], df);
            widen(wv[j], wf);
#pragma unroll
            for (int e = 0; e < 8; ++e) dot += df[e] * wf[e] * xf[e];
        }
        dot = wave_sum(dot);
        if (lane == 0) wsum[par][wave] = dot;
        // Workgroup barrier that waits for the LDS write only: a full __syncthreads() would also wait for the
        // next row's loads, which are meant to stay in flight across it.  The other parity's slots are free
        // again: everybody read them before this barrier.
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        dot = (wsum[par][0] + wsum[par][1]) + (wsum[par][2] + wsum[par][3]);
        const float coef = r * r * r * dot / (float)C;
        __bf16* dxr = dx + row * C;
#pragma unroll
        for (int j = 0; j < NVT; ++j) {
            const int c0 = (j * 256 + (int)threadIdx.x) * 8;
            float xf[8], df[8], wf[8], o[8];
            widen(xv[j], xf);
            widen(dv[j], df);
            widen(wv[j], wf);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                o[e] = df[e] * wf[e] * r - xf[e] * coef;
                dwacc[j][e] += df[e] * xf[e] * r;
            }
            if (c0 < C) st16(dxr + c0, narrow(o));
        }
    }
    float* prow = part + (size_t)blockIdx.x * C;
#pragma unroll
    for (int j = 0; j < NVT; ++j) {
        const int c0 = (j * 256 + (int)threadIdx.x) * 8;
        if (c0 < C) {
            *reinterpret_cast<f32x4*>(prow + c0) = f32x4{dwacc[j][0], dwacc[j][1], dwacc[j][2], dwacc[j][3]};
            *reinterpret_cast<f32x4*>(prow + c0 + 4) = f32x4{dwacc[j][4], dwacc[j][5], dwacc[j][6], dwacc[j][7]};
        }
    }
}

// dw[c] = sum of the partial rows, in a fixed order.  A block takes 64 columns: 16 threads across (four
// columns, one 16-byte load each) by 16 thread rows; thread row k adds partial rows k, k+16, ... (all its
// loads independent, so they are in flight together), and the 16 sums are added in thread-row order
// through LDS.  Every load instruction of a wave covers whole 256-byte row segments.
__global__ __launch_bounds__(256) void rmsnorm_dw_kernel(const float* __restrict__ part, __bf16* __restrict__ dw,
                                                        int32_t n_part, int32_t C) {
    __shared__ f32x4 red[16][16];
    const int cl = threadIdx.x & 15, pl = threadIdx.x >> 4;
    const int c = blockIdx.x * 64 + cl * 4;  // C is a multiple of 8, so a quad is inside the row or outside it
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (c < C) {
#pragma unroll 8
        for (int i = pl; i < n_part; i += 16) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(part + (size_t)i * C + c);
            s += v;
        }
    }
    red[pl][cl] = s;
    __syncthreads();
    if (pl == 0 && c < C) {
        f32x4 t = red[0][cl];
#pragma unroll
        for (int k = 1; k < 16; ++k) t += red[k][cl];
        const f32x2 lo = {t[0], t[1]}, hi = {t[2], t[3]};
        uint32_t w[2] = {__builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2)),
                         __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2))};
        *reinterpret_cast<uint2*>(dw + c) = uint2{w[0], w[1]};
    }
}

// ------------------------------------------------------------------ rotary embedding
// x [T, H, D]; element i of the first half of the head dim and element i of the second half are rotated
// by the angle whose cosine and sine are cos[t, i], sin[t, i] (fp32 tables [T, D/2]); conjugate = the
// rotation by the negative angle (the gradient).  A thread takes 8 consecutive i.  out may be x itself.
__global__ __launch_bounds__(256) void rope_kernel(const __bf16* x, const float* __restrict__ cs,
                                                  const float* __restrict__ sn, __bf16* out, int64_t n_vec,
                                                  int32_t H, int32_t D, float sign) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= n_vec) return;
    const int32_t vph = D / 16;  // vectors per half head
    const int64_t th = v / vph;  // t*H + h
    const int32_t i0 = (int32_t)(v - th * vph) * 8;
    const int64_t t = th / H;
    const __bf16* p1 = x + th * D + i0;
    float a[8], b[8], c[8], s[8];
    widen(ld16(p1), a);
    widen(ld16(p1 + D / 2), b);
    const float* cp = cs + t * (D / 2) + i0;
    const float* sp_ = sn + t * (D / 2) + i0;
    *reinterpret_cast<f32x4*>(c) = *reinterpret_cast<const f32x4*>(cp);
    *reinterpret_cast<f32x4*>(c + 4) = *reinterpret_cast<const f32x4*>(cp + 4);
    *reinterpret_cast<f32x4*>(s) = *reinterpret_cast<const f32x4*>(sp_);
    *reinterpret_cast<f32x4*>(s + 4) = *reinterpret_cast<const f32x4*>(sp_ + 4);
    float o1[8], o2[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float se = sign * s[e];
        o1[e] = a[e] * c[e] - b[e] * se;
        o2[e] = b[e] * c[e] + a[e] * se;
    }
    __bf16* q1 = out + th * D + i0;
    st16(q1, narrow(o1));
    st16(q1 + D / 2, narrow(o2));
}

// ------------------------------------------------------------------ SwiGLU gate
__device__ __forceinline__ float sigmoidf(float g) { return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-g * kLog2e)); }

__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const __bf16* __restrict__ g, const __bf16* __restrict__ u,
                                                        __bf16* __restrict__ y, int64_t n_vec) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= n_vec) return;
    float gf[8], uf[8], o[8];
    widen(ld16(g + v * 8), gf);
    widen(ld16(u + v * 8), uf);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = gf[e] * sigmoidf(gf[e]) * uf[e];
    st16(y + v * 8, narrow(o));
}

__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const __bf16* __restrict__ g, const __bf16* __restrict__ u,
                                                        const __bf16* __restrict__ dy, __bf16* __restrict__ dg,
                                                        __bf16* __restrict__ du, int64_t n_vec) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= n_vec) return;
    float gf[8], uf[8], df[8], og[8], ou[8];
    widen(ld16(g + v * 8), gf);
    widen(ld16(u + v * 8), uf);
    widen(ld16(dy + v * 8), df);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float sg = sigmoidf(gf[e]);
        og[e] = df[e] * uf[e] * sg * (1.0f + gf[e] * (1.0f - sg));
        ou[e] = df[e] * gf[e] * sg;
    }
    st16(dg + v * 8, narrow(og));
    st16(du + v * 8, narrow(ou));
}

inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }
#ifndef SP_RMS_BWD_GROUPS
#define SP_RMS_BWD_GROUPS 512
#endif
constexpr int kRmsBwdGroups = SP_RMS_BWD_GROUPS;  // workgroups of the RMS-norm backward = partial rows of dw

}  // namespace

namespace sp {

int32_t rmsnorm_bwd_groups(int64_t T) { return (int32_t)(T < kRmsBwdGroups ? (T < 1 ? 1 : T) : kRmsBwdGroups); }

sp_status launch_rmsnorm_fwd(const void* x, const void* w, void* y, float* rstd, int64_t T, int32_t C, float eps,
                             hipStream_t st) {
    const dim3 grid(blocks_for(T, 4)), block(256);
    const int nv = (C + 511) / 512;
#define SP_RMS_FWD(NV) hipLaunchKernelGGL((rmsnorm_fwd_kernel<NV>), grid, block, 0, st, (const __bf16*)x, (const __bf16*)w, (__bf16*)y, rstd, T, C, eps)
    if (nv <= 1) SP_RMS_FWD(1); else if (nv <= 2) SP_RMS_FWD(2); else if (nv <= 4) SP_RMS_FWD(4);
    else if (nv <= 8) SP_RMS_FWD(8); else if (nv <= 16) SP_RMS_FWD(16); else return SP_ERR_UNSUPPORTED;
#undef SP_RMS_FWD
    return launch_status();
}

sp_status launch_rmsnorm_bwd(const void* x, const void* w, const float* rstd, const void* dy, void* dx, void* dw,
                             float* part, int64_t T, int32_t C, hipStream_t st) {
    const int32_t groups = rmsnorm_bwd_groups(T);
    const dim3 grid(groups), block(256);
    const int nv = (C + 2047) / 2048;
#define SP_RMS_BWD(NV) hipLaunchKernelGGL((rmsnorm_bwd_kernel<NV>), grid, block, 0, st, (const __bf16*)x, (const __bf16*)w, rstd, (const __bf16*)dy, (__bf16*)dx, part, T, C)
    if (nv <= 1) SP_RMS_BWD(1); else if (nv <= 2) SP_RMS_BWD(2); else if (nv <= 4) SP_RMS_BWD(4); else return SP_ERR_UNSUPPORTED;
#undef SP_RMS_BWD
    if (launch_status() != SP_OK) return SP_ERR_LAUNCH;
    hipLaunchKernelGGL(rmsnorm_dw_kernel, dim3(blocks_for(C, 64)), dim3(256), 0, st, part, (__bf16*)dw, groups, C);
    return launch_status();
}

sp_status launch_rope(const void* x, const float* cs, const float* sn, void* out, int64_t T, int32_t H, int32_t D,
                      bool conjugate, hipStream_t st) {
    const int64_t n_vec = T * H * (D / 16);
    if ((n_vec + 255) / 256 > 0x7fffffff) return SP_ERR_SHAPE;
    hipLaunchKernelGGL(rope_kernel, dim3(blocks_for(n_vec, 256)), dim3(256), 0, st, (const __bf16*)x, cs, sn, (__bf16*)out,
                       n_vec, H, D, conjugate ? -1.0f : 1.0f);
    return launch_status();
}

sp_status launch_swiglu_fwd(const void* g, const void* u, void* y, int64_t n, hipStream_t st) {
    const int64_t n_vec = n / 8;
    if ((n_vec + 255) / 256 > 0x7fffffff) return SP_ERR_SHAPE;
    hipLaunchKernelGGL(swiglu_fwd_kernel, dim3(blocks_for(n_vec, 256)), dim3(256), 0, st, (const __bf16*)g, (const __bf16*)u,
                       (__bf16*)y, n_vec);
    return launch_status();
}

sp_status launch_swiglu_bwd(const void* g, const void* u, const void* dy, void* dg, void* du, int64_t n, hipStream_t st) {
    const int64_t n_vec = n / 8;
    if ((n_vec + 255) / 256 > 0x7fffffff) return SP_ERR_SHAPE;
    hipLaunchKernelGGL(swiglu_bwd_kernel, dim3(blocks_for(n_vec, 256)), dim3(256), 0, st, (const __bf16*)g, (const __bf16*)u,
                       (const __bf16*)dy, (__bf16*)dg, (__bf16*)du, n_vec);
    return launch_status();
}

}  // namespace sp
