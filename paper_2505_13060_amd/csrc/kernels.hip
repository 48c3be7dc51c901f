// HIP kernels of libampsens for gfx950 (MI355X): absmax scan, FP8 fake quantisation, and the
// fused sensitivity pass
//     E_f = sum_k xdot_k^2 (x_k - xtilde_k)^2   (first-order Taylor term of Sec. 2.2 of the paper,
//                                                 with the actual FP8 rounding error)
//     A   = sum_k xdot_k^2 x_k^2                (the sensitivity ||z (.) zdot||^2 of Sec. 2.2)
// The pass is bound by the HBM read of x and xdot (4 bytes per element pair); there is no
// contraction, so no MFMA.  Per pair and format the ALU work is one multiply by the reciprocal
// scale, a clamp, half a packed convert to FP8 (gfx950's OCP conversion instructions), half a
// packed convert back, one FMA for the error and a multiply + FMA for the sum.
//
// Build with -ffp-contract=off: the multiply that decides an FP8 code must stay a plain fp32
// multiply; every fusion that is wanted is written as fmaf.
#include "internal.h"
#include "walk.h"

namespace ampsens {
namespace {

typedef float float2_t __attribute__((ext_vector_type(2)));
typedef const uint16_t __attribute__((address_space(1)))* gptr16_t;   // global address space
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));             // one 128-bit load
typedef const u32x4 __attribute__((address_space(1)))* gptr128_t;

template <int FMT> struct Fp8;
template <> struct Fp8<0> {                       // OCP E4M3
    static constexpr float kMax = 448.0f;
    static __device__ __forceinline__ int pack(float a, float b, int old, bool hi) {
        return hi ? __builtin_amdgcn_cvt_pk_fp8_f32(a, b, old, true)
                  : __builtin_amdgcn_cvt_pk_fp8_f32(a, b, old, false);
    }
    static __device__ __forceinline__ float2_t unpack(int pk, bool hi) {
        return hi ? __builtin_amdgcn_cvt_pk_f32_fp8(pk, true)
                  : __builtin_amdgcn_cvt_pk_f32_fp8(pk, false);
    }
};
template <> struct Fp8<1> {                       // OCP E5M2
    static constexpr float kMax = 57344.0f;
    static __device__ __forceinline__ int pack(float a, float b, int old, bool hi) {
        return hi ? __builtin_amdgcn_cvt_pk_bf8_f32(a, b, old, true)
                  : __builtin_amdgcn_cvt_pk_bf8_f32(a, b, old, false);
    }
    static __device__ __forceinline__ float2_t unpack(int pk, bool hi) {
        return hi ? __builtin_amdgcn_cvt_pk_f32_bf8(pk, true)
                  : __builtin_amdgcn_cvt_pk_f32_bf8(pk, false);
    }
};

template <int FMT>
__device__ __forceinline__ float clamp_fmax(float y) {
    return __builtin_amdgcn_fmed3f(y, -Fp8<FMT>::kMax, Fp8<FMT>::kMax);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        uint32_t w = (uint32_t)__shfl_xor((int)v, o);
        v = v > w ? v : w;
    }
    return v;
}

// Fetch x[e + j] for jlo <= j < jhi one element at a time, zero elsewhere, packed like a
// 128-bit load would deliver them.
__device__ __forceinline__ u32x4 gather8(gptr16_t p, int64_t e, int jlo, int jhi) {
    uint32_t h[kVec];
#pragma unroll
    for (int j = 0; j < kVec; ++j) h[j] = (j >= jlo && j < jhi) ? (uint32_t)p[e + j] : 0u;
    u32x4 v = {h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    return v;
}

// ---- the fused sensitivity pass --------------------------------------------------------------

template <int NF, int F0, int F1>
struct SensCtx {
    gptr16_t x;
    gptr16_t g;
    float inv[NF], scale[NF];
    float E[NF];
    float A;
    int pk[NF];                                    // conversion scratch, carried so that the packed
                                                   // converts never need a cleared destination

    // Four elements (two input words) of one format.
    template <int F>
    __device__ __forceinline__ void one_format(const float (&xv)[4], const float (&gv)[4], float iv,
                                               float sc, float& Ef, int& p) {
        const float y0 = clamp_fmax<F>(xv[0] * iv);
        const float y1 = clamp_fmax<F>(xv[1] * iv);
        const float y2 = clamp_fmax<F>(xv[2] * iv);
        const float y3 = clamp_fmax<F>(xv[3] * iv);
        p = Fp8<F>::pack(y0, y1, p, false);
        p = Fp8<F>::pack(y2, y3, p, true);
        const float2_t q01 = Fp8<F>::unpack(p, false);
        const float2_t q23 = Fp8<F>::unpack(p, true);
        const float e0 = fmaf(-q01.x, sc, xv[0]);    // x - q*scale, one rounding
        const float e1 = fmaf(-q01.y, sc, xv[1]);
        const float e2 = fmaf(-q23.x, sc, xv[2]);
        const float e3 = fmaf(-q23.y, sc, xv[3]);
        const float t0 = gv[0] * e0, t1 = gv[1] * e1, t2 = gv[2] * e2, t3 = gv[3] * e3;
        Ef = fmaf(t0, t0, Ef);
        Ef = fmaf(t1, t1, Ef);
        Ef = fmaf(t2, t2, Ef);
        Ef = fmaf(t3, t3, Ef);
    }

    __device__ __forceinline__ void quad(uint32_t xw0, uint32_t xw1, uint32_t gw0, uint32_t gw1) {
        const float xv[4] = {bf16_lo(xw0), bf16_hi(xw0), bf16_lo(xw1), bf16_hi(xw1)};
        const float gv[4] = {bf16_lo(gw0), bf16_hi(gw0), bf16_lo(gw1), bf16_hi(gw1)};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = gv[j] * xv[j];
            A = fmaf(a, a, A);
        }
        one_format<F0>(xv, gv, inv[0], scale[0], E[0], pk[0]);
        if constexpr (NF > 1) one_format<F1>(xv, gv, inv[1], scale[1], E[1], pk[1]);
    }

    __device__ __forceinline__ void vec(const u32x4& xv, const u32x4& gv) {
        quad(xv.x, xv.y, gv.x, gv.y);
        quad(xv.z, xv.w, gv.z, gv.w);
    }

    template <int U>
    __device__ __forceinline__ void full(int64_t e, int64_t stride) {
        u32x4 xr[U], gr[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            xr[k] = *reinterpret_cast<gptr128_t>(x + e + k * stride);
            gr[k] = *reinterpret_cast<gptr128_t>(g + e + k * stride);
        }
#pragma unroll
        for (int k = 0; k < U; ++k) vec(xr[k], gr[k]);
    }

    __device__ __forceinline__ void partial(int64_t e, int jlo, int jhi) {
        const u32x4 xv = gather8(x, e, jlo, jhi);
        const u32x4 gv = gather8(g, e, jlo, jhi);
        vec(xv, gv);                               // absent elements are (0, 0): they add exactly 0
    }
};

template <int NF, int F0, int F1>
__global__ __launch_bounds__(kWG) void sens_kernel(const WorkUnit* __restrict__ units,
                                                   const uint32_t* __restrict__ chunk_begin,
                                                   uint32_t n_units, uint32_t n_chunks,
                                                   float* __restrict__ partials) {
    __shared__ float red[2][kWG / 64][NF + 1];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    uint32_t it = 0;
    for (uint32_t c = blockIdx.x; c < n_chunks; c += gridDim.x, ++it) {
        const uint32_t ui = find_unit(chunk_begin, n_units, c);
        const WorkUnit u = units[ui];
        SensCtx<NF, F0, F1> ctx;
        ctx.x = (gptr16_t)u.x;
        ctx.g = (gptr16_t)u.dx;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            ctx.inv[f] = u.inv[f];
            ctx.scale[f] = u.scale[f];
            ctx.E[f] = 0.0f;
            ctx.pk[f] = 0;
        }
        ctx.A = 0.0f;
        walk_chunk(u, c - chunk_begin[ui], tid, ctx);

        float v[NF + 1];
#pragma unroll
        for (int f = 0; f < NF; ++f) v[f] = wave_sum(ctx.E[f]);
        v[NF] = wave_sum(ctx.A);
        float (*slot)[NF + 1] = red[it & 1];
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k <= NF; ++k) slot[wave][k] = v[k];
        }
        __syncthreads();
        // Two alternating slots and one barrier per chunk: a wave can reach the writes of
        // chunk it+2 only after every wave passed the barrier of chunk it+1, hence after
        // thread 0 finished reading the slot of chunk it.
        if (tid == 0) {
#pragma unroll
            for (int k = 0; k <= NF; ++k)
                partials[(size_t)c * (NF + 1) + k] =
                    (slot[0][k] + slot[1][k]) + (slot[2][k] + slot[3][k]);
        }
    }
}

// One wave per unit: fixed-order fp64 sum of the unit's chunk partials.
template <int NF>
__global__ __launch_bounds__(kWG) void sens_finalize_kernel(const WorkUnit* __restrict__ units,
                                                            const uint32_t* __restrict__ chunk_begin,
                                                            uint32_t n_units,
                                                            const float* __restrict__ partials,
                                                            float* __restrict__ out) {
    const uint32_t ui = blockIdx.x * (kWG / 64) + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (ui >= n_units) return;
    const uint32_t c0 = chunk_begin[ui], c1 = chunk_begin[ui + 1];
    double acc[NF + 1];
#pragma unroll
    for (int k = 0; k <= NF; ++k) acc[k] = 0.0;
    for (uint32_t c = c0 + lane; c < c1; c += 64) {
#pragma unroll
        for (int k = 0; k <= NF; ++k) acc[k] += (double)partials[(size_t)c * (NF + 1) + k];
    }
#pragma unroll
    for (int k = 0; k <= NF; ++k) acc[k] = wave_sum(acc[k]);
    if (lane == 0) {
        const uint32_t o = units[ui].out;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            out[o + 4 * f] = (float)acc[f];
            out[o + 4 * f + 1] = (float)acc[NF];
        }
    }
}

// ---- absmax ---------------------------------------------------------------------------------

struct AbsmaxCtx {
    gptr16_t x;
    uint32_t m;                                     // running max of (bits & 0x7FFF)

    __device__ __forceinline__ void word(uint32_t w) {
        const uint32_t lo = w & 0x7FFFu, hi = (w >> 16) & 0x7FFFu;
        m = m > lo ? m : lo;
        m = m > hi ? m : hi;
    }
    __device__ __forceinline__ void vec(const u32x4& v) { word(v.x); word(v.y); word(v.z); word(v.w); }

    template <int U>
    __device__ __forceinline__ void full(int64_t e, int64_t stride) {
        u32x4 xr[U];
#pragma unroll
        for (int k = 0; k < U; ++k) xr[k] = *reinterpret_cast<gptr128_t>(x + e + k * stride);
#pragma unroll
        for (int k = 0; k < U; ++k) vec(xr[k]);
    }
    __device__ __forceinline__ void partial(int64_t e, int jlo, int jhi) { vec(gather8(x, e, jlo, jhi)); }
};

__global__ __launch_bounds__(kWG) void absmax_kernel(const WorkUnit* __restrict__ units,
                                                     const uint32_t* __restrict__ chunk_begin,
                                                     uint32_t n_units, uint32_t n_chunks,
                                                     uint32_t* __restrict__ maxbits) {
    const int tid = threadIdx.x;
    for (uint32_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const uint32_t ui = find_unit(chunk_begin, n_units, c);
        const WorkUnit u = units[ui];
        AbsmaxCtx ctx;
        ctx.x = (gptr16_t)u.x;
        ctx.m = 0;
        walk_chunk(u, c - chunk_begin[ui], tid, ctx);
        const uint32_t m = wave_max(ctx.m);
        // integer max is exact and order-free, so an atomic keeps the result deterministic
        if ((tid & 63) == 0 && m != 0) atomicMax(&maxbits[u.out], m);
    }
}

__device__ __forceinline__ float fmax_of(int fmt) { return fmt == 0 ? 448.0f : 57344.0f; }

__global__ void absmax_finalize_kernel(const uint32_t* __restrict__ maxbits, int n_tensors,
                                       int n_fmts, int fmt0, int fmt1, float* __restrict__ amax_out,
                                       float* __restrict__ scale_out, float* __restrict__ inv_out,
                                       uint32_t* __restrict__ flags_out) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_tensors) return;
    const uint32_t bits = maxbits[t];
    const float amax = __uint_as_float(bits << 16);
    amax_out[t] = amax;
    flags_out[t] = bits >= 0x7F80u ? 1u : 0u;
    for (int f = 0; f < n_fmts; ++f) {
        const float fm = fmax_of(f == 0 ? fmt0 : fmt1);
        float scale = 1.0f, inv = 1.0f;
        if (amax != 0.0f) {
            scale = amax / fm;                      // correctly rounded fp32 divisions
            inv = fm / amax;
            if (__builtin_isinf(inv)) { scale = 1.0f; inv = 1.0f; }
        }
        scale_out[t * n_fmts + f] = scale;
        inv_out[t * n_fmts + f] = inv;
    }
}

// ---- standalone fake quantisation -------------------------------------------------------------

template <int FMT>
__global__ __launch_bounds__(kWG) void fake_quant_kernel(const uint16_t* __restrict__ x, int64_t n,
                                                         float scale, float inv,
                                                         uint8_t* __restrict__ codes,
                                                         float* __restrict__ deq, int vec_ok) {
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t gsz = (int64_t)gridDim.x * blockDim.x;
    const int64_t nvec = vec_ok ? n / kVec : 0;
    for (int64_t v = gtid; v < nvec; v += gsz) {
        const uint4 xv = reinterpret_cast<const uint4*>(x)[v];
        const uint32_t w[4] = {xv.x, xv.y, xv.z, xv.w};
        int pk[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float y0 = clamp_fmax<FMT>(bf16_lo(w[2 * h]) * inv);
            const float y1 = clamp_fmax<FMT>(bf16_hi(w[2 * h]) * inv);
            const float y2 = clamp_fmax<FMT>(bf16_lo(w[2 * h + 1]) * inv);
            const float y3 = clamp_fmax<FMT>(bf16_hi(w[2 * h + 1]) * inv);
            int p = Fp8<FMT>::pack(y0, y1, 0, false);
            pk[h] = Fp8<FMT>::pack(y2, y3, p, true);
        }
        reinterpret_cast<uint2*>(codes)[v] = make_uint2((uint32_t)pk[0], (uint32_t)pk[1]);
        if (deq) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float2_t a = Fp8<FMT>::unpack(pk[h], false);
                const float2_t b = Fp8<FMT>::unpack(pk[h], true);
                reinterpret_cast<float4*>(deq)[2 * v + h] =
                    make_float4(a.x * scale, a.y * scale, b.x * scale, b.y * scale);
            }
        }
    }
    for (int64_t i = nvec * kVec + gtid; i < n; i += gsz) {
        const float y = clamp_fmax<FMT>(__uint_as_float((uint32_t)x[i] << 16) * inv);
        const int p = Fp8<FMT>::pack(y, 0.0f, 0, false);
        codes[i] = (uint8_t)(p & 0xFF);
        if (deq) deq[i] = Fp8<FMT>::unpack(p, false).x * scale;
    }
}

template <int NF>
hipError_t launch_sens_nf(int fmt0, int fmt1, dim3 grid, hipStream_t stream, const WorkUnit* units,
                          const uint32_t* cb, uint32_t n_units, uint32_t n_chunks, float* partials) {
    if constexpr (NF == 1) {
        if (fmt0 == 0) hipLaunchKernelGGL((sens_kernel<1, 0, 0>), grid, dim3(kWG), 0, stream, units, cb, n_units, n_chunks, partials);
        else hipLaunchKernelGGL((sens_kernel<1, 1, 1>), grid, dim3(kWG), 0, stream, units, cb, n_units, n_chunks, partials);
    } else {
        if (fmt0 == 0 && fmt1 == 0) hipLaunchKernelGGL((sens_kernel<2, 0, 0>), grid, dim3(kWG), 0, stream, units, cb, n_units, n_chunks, partials);
        else if (fmt0 == 0 && fmt1 == 1) hipLaunchKernelGGL((sens_kernel<2, 0, 1>), grid, dim3(kWG), 0, stream, units, cb, n_units, n_chunks, partials);
        else if (fmt0 == 1 && fmt1 == 0) hipLaunchKernelGGL((sens_kernel<2, 1, 0>), grid, dim3(kWG), 0, stream, units, cb, n_units, n_chunks, partials);
        else hipLaunchKernelGGL((sens_kernel<2, 1, 1>), grid, dim3(kWG), 0, stream, units, cb, n_units, n_chunks, partials);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_absmax(const WorkUnit* d_units, const uint32_t* d_chunk_begin, uint32_t n_units,
                         uint32_t n_chunks, uint32_t* d_maxbits, int grid, hipStream_t stream) {
    hipLaunchKernelGGL(absmax_kernel, dim3(grid), dim3(kWG), 0, stream, d_units, d_chunk_begin,
                       n_units, n_chunks, d_maxbits);
    return hipGetLastError();
}

hipError_t launch_absmax_finalize(const uint32_t* d_maxbits, int n_tensors, int n_fmts, int fmt0,
                                  int fmt1, float* d_amax, float* d_scale, float* d_inv,
                                  uint32_t* d_flags, hipStream_t stream) {
    const int threads = 64;
    hipLaunchKernelGGL(absmax_finalize_kernel, dim3((n_tensors + threads - 1) / threads),
                       dim3(threads), 0, stream, d_maxbits, n_tensors, n_fmts, fmt0, fmt1, d_amax,
                       d_scale, d_inv, d_flags);
    return hipGetLastError();
}

hipError_t launch_fake_quant(const uint16_t* d_x, int64_t n, float scale, float inv, int fmt,
                             uint8_t* d_codes, float* d_dequant, int grid, hipStream_t stream) {
    const bool vec_ok = ((uintptr_t)d_x % 16 == 0) && ((uintptr_t)d_codes % 8 == 0) &&
                        (d_dequant == nullptr || (uintptr_t)d_dequant % 16 == 0);
    if (fmt == 0)
        hipLaunchKernelGGL(fake_quant_kernel<0>, dim3(grid), dim3(kWG), 0, stream, d_x, n, scale,
                           inv, d_codes, d_dequant, vec_ok ? 1 : 0);
    else
        hipLaunchKernelGGL(fake_quant_kernel<1>, dim3(grid), dim3(kWG), 0, stream, d_x, n, scale,
                           inv, d_codes, d_dequant, vec_ok ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_sens(const WorkUnit* d_units, const uint32_t* d_chunk_begin, uint32_t n_units,
                       uint32_t n_chunks, int n_fmts, int fmt0, int fmt1, float* d_partials,
                       int grid, hipStream_t stream) {
    if (n_fmts == 1)
        return launch_sens_nf<1>(fmt0, fmt0, dim3(grid), stream, d_units, d_chunk_begin, n_units,
                                 n_chunks, d_partials);
    return launch_sens_nf<2>(fmt0, fmt1, dim3(grid), stream, d_units, d_chunk_begin, n_units,
                             n_chunks, d_partials);
}

hipError_t launch_sens_finalize(const WorkUnit* d_units, const uint32_t* d_chunk_begin,
                                uint32_t n_units, int n_fmts, const float* d_partials,
                                float* d_out, hipStream_t stream) {
    const dim3 grid((n_units + (kWG / 64) - 1) / (kWG / 64));
    if (n_fmts == 1)
        hipLaunchKernelGGL(sens_finalize_kernel<1>, grid, dim3(kWG), 0, stream, d_units,
                           d_chunk_begin, n_units, d_partials, d_out);
    else
        hipLaunchKernelGGL(sens_finalize_kernel<2>, grid, dim3(kWG), 0, stream, d_units,
                           d_chunk_begin, n_units, d_partials, d_out);
    return hipGetLastError();
}

}  // namespace ampsens
