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
// Streaming design: a persistent grid (as many workgroups as are resident) strides over the
// chunk list of all units of a call; chunk c is found through a device-built map (no search),
// the next chunk's map entry is fetched while the current chunk streams; operands are read
// with 128-bit non-temporal loads addressed as uniform base + lane offset; every wave reduces
// its lanes with DPP and writes its own partial (no LDS, no barrier); a second small kernel
// adds each unit's partials in a fixed order in fp64.
//
// Build with -ffp-contract=off: the multiply that decides an FP8 code must stay a plain fp32
// multiply; every fusion that is wanted is written as fmaf.
#include "internal.h"
#include "walk.h"

#include <cstring>
#include <type_traits>

#ifndef AMPSENS_W_LOAD
#define AMPSENS_W_LOAD 8
#endif

namespace ampsens {
namespace {

constexpr int kWLoad = AMPSENS_W_LOAD;       // gradient vectors of one step in flight per lane

typedef float float2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef short short2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));             // one 128-bit load
typedef const uint16_t __attribute__((address_space(1)))* gptr16_t;   // global address space
typedef const u32x4 __attribute__((address_space(1)))* gptr128_t;
typedef const float __attribute__((address_space(1)))* gptrf_t;
typedef const float2_t __attribute__((address_space(1)))* gptrf2_t;
typedef const char __attribute__((address_space(1)))* gptr8_t;

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
    // gfx950's scaled conversions.  Measured over all bf16 patterns: pack_scaled gives the code of
    // RNE(x / 2^exponent(scale)) for both elements of a packed bf16 pair, WITHOUT saturation (a quotient
    // beyond the format's range gives the NaN code); unpack_scaled gives decode(code) * 2^exponent(scale).
    static __device__ __forceinline__ short2_t pack_scaled(uint32_t xw, float scale, short2_t old, bool hi) {
        return hi ? __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(old, __builtin_bit_cast(bf16x2_t, xw), scale, true)
                  : __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(old, __builtin_bit_cast(bf16x2_t, xw), scale, false);
    }
    static __device__ __forceinline__ float2_t unpack_scaled(uint32_t pk, float scale, bool hi) {
        return hi ? __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(pk, scale, true)
                  : __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(pk, scale, false);
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
    static __device__ __forceinline__ short2_t pack_scaled(uint32_t xw, float scale, short2_t old, bool hi) {   // overflow: the Inf code
        return hi ? __builtin_amdgcn_cvt_scalef32_pk_bf8_bf16(old, __builtin_bit_cast(bf16x2_t, xw), scale, true)
                  : __builtin_amdgcn_cvt_scalef32_pk_bf8_bf16(old, __builtin_bit_cast(bf16x2_t, xw), scale, false);
    }
    static __device__ __forceinline__ float2_t unpack_scaled(uint32_t pk, float scale, bool hi) {
        return hi ? __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(pk, scale, true)
                  : __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(pk, scale, false);
    }
};

template <int FMT>
__device__ __forceinline__ float clamp_fmax(float y) {
    return __builtin_amdgcn_fmed3f(y, -Fp8<FMT>::kMax, Fp8<FMT>::kMax);
}

// The sensitivity kernels leave the clamp to the conversion itself: while MODE.FP16_OVFL is set,
// gfx950's FP8 conversions turn a finite input beyond the format's range into the largest finite code
// (measured for every bf16 pattern as fp32 input and for fp32 values around 448 / 464 / 480 and
// 57344 / 61440 / 65536: the same code as clamping to +-FMAX first; infinities and NaN keep their own
// codes), which saves one instruction per element and format.  MODE belongs to the wave and ends with
// it; every sensitivity kernel calls this before anything else.
__device__ __forceinline__ void saturating_fp8_conversions() {
    __builtin_amdgcn_s_setreg(1 | (23 << 6) | (0 << 11), 1);       // hwreg(HW_REG_MODE, offset 23, 1 bit) = FP16_OVFL
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// ---- wave64 reductions ------------------------------------------------------------------------

// v + (v moved by a DPP pattern); rows the mask leaves out, and lanes without a source, add 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false);
    return v + __int_as_float(moved);
}

// Sum over the 64 lanes in a fixed order; the total is returned in every lane.
__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_add<0xB1, 0xF>(v);        // quad_perm [1,0,3,2]
    v = dpp_add<0x4E, 0xF>(v);        // quad_perm [2,3,0,1]
    v = dpp_add<0x141, 0xF>(v);       // row_half_mirror
    v = dpp_add<0x140, 0xF>(v);       // row_mirror: every lane of a 16-lane row holds the row sum
    v = dpp_add<0x142, 0xA>(v);       // row_bcast15 into rows 1 and 3
    v = dpp_add<0x143, 0xC>(v);       // row_bcast31 into rows 2 and 3: lane 63 holds the total
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
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

// ---- loads --------------------------------------------------------------------------------------

template <bool NT>
__device__ __forceinline__ u32x4 load128(gptr128_t p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
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

// Keep the first `tail` (1..8) bf16 elements of a vector, clear the rest.
__device__ __forceinline__ u32x4 keep_leading(u32x4 v, int tail) {
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t m = tail >= 2 * k + 2 ? 0xFFFFFFFFu : (tail == 2 * k + 1 ? 0x0000FFFFu : 0u);
        w[k] &= m;
    }
    u32x4 r = {w[0], w[1], w[2], w[3]};
    return r;
}

// ---- descriptor tables arrive as kernel arguments ------------------------------------------------
// A call's table (a few KB to a few hundred KB of unit records) is cut into pieces that travel as
// the by-value argument of this kernel: no staging buffer, no copy engine, nothing that outlives
// the call on the host, and a launch that a HIP graph can hold by value.
__global__ __launch_bounds__(kWG) void table_write_kernel(TablePiece piece, uint4* __restrict__ dst,
                                                          uint32_t n_words) {
    for (uint32_t i = threadIdx.x; i < n_words; i += kWG) dst[i] = piece.w[i];
}

// Records that stand for runs of units whose fields advance by fixed steps (internal.h): one
// workgroup per record, one thread per 64-bit word of the expanded units.
__global__ __launch_bounds__(64) void table_runs_kernel(TablePiece piece, uint8_t* __restrict__ table,
                                                        uint32_t off_schedule) {
    const TableRun& R = reinterpret_cast<const TableRun*>(&piece)[blockIdx.x];
    constexpr uint32_t kWords = 8 + 2;                 // unit, schedule
    for (uint32_t i = threadIdx.x; i < R.count * kWords; i += 64) {
        const uint32_t k = i / kWords, w = i % kWords;
        const uint64_t u = (uint64_t)R.first_unit + (uint64_t)k * R.stride;
        if (w < 8)
            reinterpret_cast<uint64_t*>(table)[u * 8 + w] = R.unit[w] + (uint64_t)k * R.unit_step[w];
        else
            reinterpret_cast<uint64_t*>(table + off_schedule)[u * 2 + (w - 8)] =
                R.sched[w - 8] + (uint64_t)k * R.sched_step[w - 8];
    }
}

__global__ __launch_bounds__(64) void table_literals_kernel(TablePiece piece, uint8_t* __restrict__ table,
                                                            uint32_t off_schedule) {
    const TableLiteral& L = reinterpret_cast<const TableLiteral*>(&piece)[blockIdx.x];
    const uint32_t w = threadIdx.x;
    const uint64_t u = L.unit_index;
    if (w < 8)
        reinterpret_cast<uint64_t*>(table)[u * 8 + w] = L.unit[w];
    else if (w < 10)
        reinterpret_cast<uint64_t*>(table + off_schedule)[u * 2 + (w - 8)] = L.sched[w - 8];
}

// ---- prepare: the static part of a call (once per set-up) ----------------------------------------
// Unit records in the form the streaming kernels read, and the chunk map: for every schedule
// position its unit, its index inside that unit and its partial slot, so that no kernel searches.
__device__ __forceinline__ void prepare_item(uint32_t i, const WorkUnit* __restrict__ units,
                                             const uint32_t* __restrict__ chunk_begin,
                                             const UnitSchedule* __restrict__ schedule, uint32_t n_units,
                                             uint32_t n_chunks, ResolvedUnit* __restrict__ runits,
                                             ChunkRef* __restrict__ map) {
    if (i < n_units) {
        const WorkUnit u = units[i];
        ResolvedUnit r;
        r.x = u.x; r.dx = u.dx; r.n = u.n; r.rows = u.rows; r.cols = u.cols; r.flags = u.flags;
        r.head = u.head; r.out = u.out; r.chunks_per_mat = u.chunks_per_mat;
        if (u.flags & kUnitRowScale) {
            r.row_inv = u.inv;
            r.row_scale = u.scale;
        } else {
            for (int f = 0; f < kMaxFormats; ++f) { r.inv[f] = 1.0f; r.scale[f] = 1.0f; }
        }
        runits[i] = r;
    }
    if (i < n_chunks) {
        const uint32_t ui = find_unit(chunk_begin, n_units, i);
        ChunkRef ref;
        ref.unit = ui;
        ref.local = i - chunk_begin[ui];
        ref.slot = i;
        ref.reserved = 0;
        const UnitSchedule sch = schedule[ui];
        if (ref.local >= sch.skip)
            map[schedule_position(sch, ref.local - sch.skip,
                                  chunk_begin[ui + 1] - chunk_begin[ui] - sch.skip)] = ref;
    }
}

__global__ __launch_bounds__(kWG) void prepare_kernel(const WorkUnit* __restrict__ units,
                                                      const uint32_t* __restrict__ chunk_begin,
                                                      const UnitSchedule* __restrict__ schedule,
                                                      uint32_t n_units, uint32_t n_chunks,
                                                      ResolvedUnit* __restrict__ runits,
                                                      ChunkRef* __restrict__ map) {
    prepare_item(blockIdx.x * blockDim.x + threadIdx.x, units, chunk_begin, schedule, n_units, n_chunks, runits, map);
}

// ---- resolve: the scales of a run (every run) ------------------------------------------------------
// Units with one scale per tensor get the values their scale pointers hold now (an absmax run on
// the same stream may just have written them); units with row scales keep their table pointers.
__device__ __forceinline__ void resolve_item(uint32_t i, const WorkUnit* __restrict__ units, int n_fmts,
                                             ResolvedUnit* __restrict__ runits) {
    const WorkUnit u = units[i];
    if (u.flags & kUnitRowScale) return;
    for (int f = 0; f < kMaxFormats; ++f) {
        const bool have = f < n_fmts && u.inv != nullptr && u.scale != nullptr;
        runits[i].inv[f] = have ? u.inv[f] : 1.0f;
        runits[i].scale[f] = have ? u.scale[f] : 1.0f;
    }
}

__global__ __launch_bounds__(kWG) void resolve_kernel(const WorkUnit* __restrict__ units, uint32_t n_units,
                                                      int n_fmts, ResolvedUnit* __restrict__ runits) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_units) resolve_item(i, units, n_fmts, runits);
}

// ---- small calls: table, prepare and (for a call that runs at once) resolve in one launch -------------
// A table that fits one piece is written, and then read back by the same single workgroup after a
// barrier: the set-up of a small call is one launch instead of two or three.  resolve_fmts > 0:
// the scales are resolved too (the caller runs the pass right after, on the same stream).
__global__ __launch_bounds__(kWG) void small_setup_kernel(TablePiece piece, uint32_t n_words, uint4* __restrict__ dst,
                                                          uint32_t off_cb, uint32_t off_schedule, uint32_t n_units,
                                                          uint32_t n_chunks, ResolvedUnit* __restrict__ runits,
                                                          ChunkRef* __restrict__ map, int resolve_fmts) {
    for (uint32_t i = threadIdx.x; i < n_words; i += kWG) dst[i] = piece.w[i];
    __threadfence_block();
    __syncthreads();
    const uint8_t* base = reinterpret_cast<const uint8_t*>(dst);
    const WorkUnit* units = reinterpret_cast<const WorkUnit*>(base);
    const uint32_t* chunk_begin = reinterpret_cast<const uint32_t*>(base + off_cb);
    const UnitSchedule* schedule = reinterpret_cast<const UnitSchedule*>(base + off_schedule);
    const uint32_t n = n_units > n_chunks ? n_units : n_chunks;
    for (uint32_t i = threadIdx.x; i < n; i += kWG)
        prepare_item(i, units, chunk_begin, schedule, n_units, n_chunks, runits, map);
    if (resolve_fmts > 0) {
        // a thread resolves the units it has just prepared itself: no second barrier
        for (uint32_t i = threadIdx.x; i < n_units; i += kWG) resolve_item(i, units, resolve_fmts, runits);
    }
}

// ---- the fused sensitivity pass --------------------------------------------------------------

// Four elements (two input words) of one format; p is conversion scratch, carried so that the
// packed converts never need a cleared destination.
template <int F>
__device__ __forceinline__ void one_format(const float (&xv)[4], const float (&gv)[4], float iv,
                                           float sc, float& Ef, int& p) {
    {
        const float y0 = xv[0] * iv, y1 = xv[1] * iv, y2 = xv[2] * iv, y3 = xv[3] * iv;   // the conversion saturates
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
}

// The same four elements when the scale is a power of two s, the reciprocal is 1 / s, and no element
// exceeds FMAX * s in magnitude (all true for scales the power-of-two rule derives from the absmax of
// the same data): the scaled conversions take the packed bf16 pair straight to its codes and the
// codes straight back to q * s, both exact, so the multiply and the clamp of the general path go away
// (16 instead of 24 operations per four elements and format).  q * s itself can be 2^128 (a value in
// bf16's top binade that rounds up), which fp32 does not hold while x - q * s does: the codes are
// taken back with sq = s / 4 and the error formed as fma(mul, q * sq, x), mul = -4, which is
// x - q * s rounded once, exactly what the general path computes.  Scales too small for a normal
// quarter (below 2^-100, where nothing can overflow) come as sq = s, mul = -1.
template <int F>
__device__ __forceinline__ void one_format_pow2(uint32_t xw0, uint32_t xw1, const float (&xv)[4],
                                                const float (&gv)[4], float sc, float sq, float mul,
                                                float& Ef, int& p) {
    short2_t c = __builtin_bit_cast(short2_t, p);
    c = Fp8<F>::pack_scaled(xw0, sc, c, false);
    c = Fp8<F>::pack_scaled(xw1, sc, c, true);
    p = __builtin_bit_cast(int, c);
    const float2_t q01 = Fp8<F>::unpack_scaled((uint32_t)p, sq, false);
    const float2_t q23 = Fp8<F>::unpack_scaled((uint32_t)p, sq, true);
    const float e0 = fmaf(mul, q01.x, xv[0]), e1 = fmaf(mul, q01.y, xv[1]);
    const float e2 = fmaf(mul, q23.x, xv[2]), e3 = fmaf(mul, q23.y, xv[3]);
    const float t0 = gv[0] * e0, t1 = gv[1] * e1, t2 = gv[2] * e2, t3 = gv[3] * e3;
    Ef = fmaf(t0, t0, Ef);
    Ef = fmaf(t1, t1, Ef);
    Ef = fmaf(t2, t2, Ef);
    Ef = fmaf(t3, t3, Ef);
}

template <int NF, int F0, int F1, bool POW2 = false>
struct SensCtx {
    static constexpr bool kRollDense = false;
    gptr16_t x;
    gptr16_t g;
    bool keep_x;                                   // x is re-read soon: ordinary caching
    float inv[NF], scale[NF];                      // POW2: inv holds the scale the codes are taken back with
    float mul;                                     // POW2 only: see one_format_pow2
    float E[NF];
    float A;
    int pk[NF];

    __device__ __forceinline__ void init(const ResolvedUnit& u) {
        x = (gptr16_t)u.x;
        g = (gptr16_t)u.dx;
        keep_x = (u.flags & kUnitKeepX) != 0;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            inv[f] = u.inv[f];
            scale[f] = u.scale[f];
            E[f] = 0.0f;
            pk[f] = 0;
        }
        mul = -1.0f;
        if constexpr (POW2) {                          // one multiplier for both formats
            const bool roomy = scale[0] >= 0x1p-100f && scale[NF - 1] >= 0x1p-100f;
            mul = roomy ? -4.0f : -1.0f;
#pragma unroll
            for (int f = 0; f < NF; ++f) inv[f] = roomy ? scale[f] * 0.25f : scale[f];
        }
        A = 0.0f;
    }
    __device__ __forceinline__ void begin_dense(int64_t, int) {}
    __device__ __forceinline__ void set_row(int64_t) {}

    __device__ __forceinline__ void quad(uint32_t xw0, uint32_t xw1, uint32_t gw0, uint32_t gw1) {
        const float xv[4] = {bf16_lo(xw0), bf16_hi(xw0), bf16_lo(xw1), bf16_hi(xw1)};
        const float gv[4] = {bf16_lo(gw0), bf16_hi(gw0), bf16_lo(gw1), bf16_hi(gw1)};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = gv[j] * xv[j];
            A = fmaf(a, a, A);
        }
        if constexpr (POW2) {
            one_format_pow2<F0>(xw0, xw1, xv, gv, scale[0], inv[0], mul, E[0], pk[0]);
            if constexpr (NF > 1) one_format_pow2<F1>(xw0, xw1, xv, gv, scale[1], inv[1], mul, E[1], pk[1]);
        } else {
            one_format<F0>(xv, gv, inv[0], scale[0], E[0], pk[0]);
            if constexpr (NF > 1) one_format<F1>(xv, gv, inv[1], scale[1], E[1], pk[1]);
        }
    }

    __device__ __forceinline__ void vec(const u32x4& xv, const u32x4& gv) {
        quad(xv.x, xv.y, gv.x, gv.y);
        quad(xv.z, xv.w, gv.z, gv.w);
    }

    template <int U>
    __device__ __forceinline__ void full(int64_t eu, int le, int64_t stride) {
        // uniform base (scalar registers) + this lane's vector index: one address VGPR in all
        const gptr128_t bx = reinterpret_cast<gptr128_t>(x + eu);
        const gptr128_t bg = reinterpret_cast<gptr128_t>(g + eu);
        const int lv = le / kVec;
        const int64_t sv = stride / kVec;
        u32x4 xr[U], gr[U];
        if (keep_x) {
#pragma unroll
            for (int k = 0; k < U; ++k) xr[k] = load128<false>(bx + k * sv + lv);
        } else {
#pragma unroll
            for (int k = 0; k < U; ++k) xr[k] = load128<true>(bx + k * sv + lv);
        }
#pragma unroll
        for (int k = 0; k < U; ++k) gr[k] = load128<true>(bg + k * sv + lv);
#pragma unroll
        for (int k = 0; k < U; ++k) vec(xr[k], gr[k]);
    }

    template <int U>
    __device__ __forceinline__ void full_masked(int64_t e, int stride, int count, int tail) {
        const gptr128_t px = reinterpret_cast<gptr128_t>(x + e);
        const gptr128_t pg = reinterpret_cast<gptr128_t>(g + e);
        const int sv = stride / kVec;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        u32x4 xr[U], gr[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            xr[k] = k < count ? load128<true>(px + k * sv) : zero;
            gr[k] = k < count ? load128<true>(pg + k * sv) : zero;
        }
        if (tail < kVec) {
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (k == count - 1) { xr[k] = keep_leading(xr[k], tail); gr[k] = keep_leading(gr[k], tail); }
        }
#pragma unroll
        for (int k = 0; k < U; ++k)
            if (k < count) vec(xr[k], gr[k]);
    }

    __device__ __forceinline__ void partial(int64_t e, int jlo, int jhi) {
        const u32x4 xv = gather8(x, e, jlo, jhi);
        const u32x4 gv = gather8(g, e, jlo, jhi);
        vec(xv, gv);                               // absent elements are (0, 0): they add exactly 0
    }
};

// The same pass with one scale per row (per-token activations, per-channel weights, rows of a
// BGEMM operand).  Scales come from [rows][NF] tables.  Three ways to know a vector's row:
//   dense, rows made of whole vectors: a RowCursor follows the thread's strided walk and the
//       scales of every vector are fetched (they sit in L1/L2: a row's entry serves row_len/8 vectors);
//   causal: the walker names the row of the vectors that follow, its scales are fetched once;
//   dense, rows not made of whole vectors: element by element, one division per element (slow,
//       only for odd row lengths or misaligned buffers).
// Only units with row scales reach this context; it is the general one (any row length).
template <int NF, int F0, int F1>
struct SensRowCtx {
    static constexpr bool kRollDense = false;
    enum Mode { kRow, kCursor, kElem };
    gptr16_t x;
    gptr16_t g;
    bool keep_x;
    gptrf_t ri;                                    // inv[row][NF]
    gptrf_t rs;                                    // scale[row][NF]
    int32_t row_len;
    Mode mode;
    RowCursor cur;
    float inv[NF], scale[NF];                      // kRow: the current row's
    float E[NF];
    float A;
    int pk[NF];

    // Row is a 32- or 64-bit index: the walks of a dense unit stay below 2^31 rows and then the
    // table is addressed as uniform base + 32-bit offset.
    template <class Row>
    __device__ __forceinline__ void load_row(Row row, float (&iv)[NF], float (&sc)[NF]) const {
        if constexpr (NF == 2) {
            const float2_t a = *reinterpret_cast<gptrf2_t>(ri + row * 2);
            const float2_t b = *reinterpret_cast<gptrf2_t>(rs + row * 2);
            iv[0] = a.x; iv[1] = a.y; sc[0] = b.x; sc[1] = b.y;
        } else {
            iv[0] = ri[row];
            sc[0] = rs[row];
        }
    }
    __device__ __forceinline__ void init(const ResolvedUnit& u) {
        x = (gptr16_t)u.x;
        g = (gptr16_t)u.dx;
        keep_x = (u.flags & kUnitKeepX) != 0;
        ri = (gptrf_t)u.row_inv;
        rs = (gptrf_t)u.row_scale;
        row_len = u.cols;
#pragma unroll
        for (int f = 0; f < NF; ++f) { E[f] = 0.0f; pk[f] = 0; inv[f] = 1.0f; scale[f] = 1.0f; }
        A = 0.0f;
        if (u.flags & kUnitCausal) mode = kRow;
        else mode = (u.flags & kUnitScalar) ? kElem : kCursor;
    }
    __device__ __forceinline__ void begin_dense(int64_t e0, int le) {
        if (mode == kCursor) cur.begin(e0, le, kWG * kVec, row_len);
    }
    __device__ __forceinline__ void set_row(int64_t row) { load_row(row, inv, scale); }

    __device__ __forceinline__ void quad(uint32_t xw0, uint32_t xw1, uint32_t gw0, uint32_t gw1,
                                         const float (&iv)[NF], const float (&sc)[NF]) {
        const float xv[4] = {bf16_lo(xw0), bf16_hi(xw0), bf16_lo(xw1), bf16_hi(xw1)};
        const float gv[4] = {bf16_lo(gw0), bf16_hi(gw0), bf16_lo(gw1), bf16_hi(gw1)};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = gv[j] * xv[j];
            A = fmaf(a, a, A);
        }
        one_format<F0>(xv, gv, iv[0], sc[0], E[0], pk[0]);
        if constexpr (NF > 1) one_format<F1>(xv, gv, iv[1], sc[1], E[1], pk[1]);
    }
    __device__ __forceinline__ void vec(const u32x4& xv, const u32x4& gv, const float (&iv)[NF],
                                        const float (&sc)[NF]) {
        quad(xv.x, xv.y, gv.x, gv.y, iv, sc);
        quad(xv.z, xv.w, gv.z, gv.w, iv, sc);
    }
    // One element with the scales of its own row.
    __device__ __forceinline__ void elem(uint32_t xb, uint32_t gb, const float (&iv)[NF], const float (&sc)[NF]) {
        const float xf = __uint_as_float(xb << 16), gf = __uint_as_float(gb << 16);
        const float a = gf * xf;
        A = fmaf(a, a, A);
        {
            const int p = Fp8<F0>::pack(xf * iv[0], 0.0f, 0, false);
            const float t = gf * fmaf(-Fp8<F0>::unpack(p, false).x, sc[0], xf);
            E[0] = fmaf(t, t, E[0]);
        }
        if constexpr (NF > 1) {
            const int p = Fp8<F1>::pack(xf * iv[1], 0.0f, 0, false);
            const float t = gf * fmaf(-Fp8<F1>::unpack(p, false).x, sc[1], xf);
            E[1] = fmaf(t, t, E[1]);
        }
    }

    template <int U>
    __device__ __forceinline__ void full(int64_t eu, int le, int64_t stride) {
        const gptr128_t bx = reinterpret_cast<gptr128_t>(x + eu);
        const gptr128_t bg = reinterpret_cast<gptr128_t>(g + eu);
        const int lv = le / kVec;
        const int64_t sv = stride / kVec;
        u32x4 xr[U], gr[U];
        if (keep_x) {
#pragma unroll
            for (int k = 0; k < U; ++k) xr[k] = load128<false>(bx + k * sv + lv);
        } else {
#pragma unroll
            for (int k = 0; k < U; ++k) xr[k] = load128<true>(bx + k * sv + lv);
        }
#pragma unroll
        for (int k = 0; k < U; ++k) gr[k] = load128<true>(bg + k * sv + lv);
        // one arithmetic path; only the source of the scales differs
        float iv[U][NF], sc[U][NF];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            if (mode == kCursor) {
                load_row((uint32_t)cur.row, iv[k], sc[k]);
                cur.advance();
            } else {
#pragma unroll
                for (int f = 0; f < NF; ++f) { iv[k][f] = inv[f]; sc[k][f] = scale[f]; }
            }
        }
#pragma unroll
        for (int k = 0; k < U; ++k) vec(xr[k], gr[k], iv[k], sc[k]);
        // keep the scheduler from pulling the next group's loads (and their scales) above this
        // group's arithmetic: the registers do not allow more than one group in flight
        __builtin_amdgcn_sched_barrier(0);
    }

    template <int U>
    __device__ __forceinline__ void full_masked(int64_t e, int stride, int count, int tail) {
        const gptr128_t px = reinterpret_cast<gptr128_t>(x + e);
        const gptr128_t pg = reinterpret_cast<gptr128_t>(g + e);
        const int sv = stride / kVec;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        u32x4 xr[U], gr[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            xr[k] = k < count ? load128<true>(px + k * sv) : zero;
            gr[k] = k < count ? load128<true>(pg + k * sv) : zero;
        }
        if (tail < kVec) {
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (k == count - 1) { xr[k] = keep_leading(xr[k], tail); gr[k] = keep_leading(gr[k], tail); }
        }
#pragma unroll
        for (int k = 0; k < U; ++k)
            if (k < count) vec(xr[k], gr[k], inv, scale);
    }

    __device__ __forceinline__ void partial(int64_t e, int jlo, int jhi) {
        if (mode == kElem) {
            elements(e, jlo, jhi);
            return;
        }
        const u32x4 xv = gather8(x, e, jlo, jhi);
        const u32x4 gv = gather8(g, e, jlo, jhi);
        float iv[NF], sc[NF];
        if (mode == kCursor) {
            load_row((uint32_t)cur.row, iv, sc);
            cur.advance();
        } else {
#pragma unroll
            for (int f = 0; f < NF; ++f) { iv[f] = inv[f]; sc[f] = scale[f]; }
        }
        vec(xv, gv, iv, sc);
    }

    // Rows that are not made of whole vectors: every element looks its row up by division.  Kept
    // out of line: it is the rare path and must not cost the others registers.
    __device__ __noinline__ void elements(int64_t e, int jlo, int jhi) {
        for (int j = jlo; j < jhi; ++j) {
            float iv[NF], sc[NF];
            load_row(row_len > 0 ? (e + j) / row_len : (int64_t)0, iv, sc);
            elem(x[e + j], g[e + j], iv, sc);
        }
    }
};

// Row scales for units whose rows hold at least 512 elements (or a power of two below that, or
// aligned causal units): the 64 lanes of a wave cover 512 contiguous elements per vector step, so a
// step meets at most two long rows, or a whole number of short ones.
// The wave follows its own position with a cursor in scalar registers and fetches the scales of
// those rows through the scalar cache; steps that lie inside one row (all of them when the row
// length is a multiple of 512) use them as scalar operands, the others select per lane.  Causal
// units: a lane stays in one row per band and fetches that row's scales once.
template <int NF, int F0, int F1, bool SHORT>
struct SensWaveRowCtx {
    static constexpr bool kRollDense = true;
    gptr16_t x;
    gptr16_t g;
    bool keep_x;
    gptrf_t ri;
    gptrf_t rs;
    int32_t row_len, last_row;
    int sub_shift;                                 // >= 0: rows of 8 << sub_shift < 512 elements
    bool causal;
    int lane;
    RowCursor cur;                                 // of the wave's first lane; uniform over the wave
    float inv[NF], scale[NF];                      // causal: of the lane's current row
    float E[NF];
    float A;
    int pk[NF];

    __device__ __forceinline__ void init(const ResolvedUnit& u) {
        x = (gptr16_t)u.x;
        g = (gptr16_t)u.dx;
        keep_x = (u.flags & kUnitKeepX) != 0;
        ri = (gptrf_t)u.row_inv;
        rs = (gptrf_t)u.row_scale;
        row_len = u.cols;
        causal = (u.flags & kUnitCausal) != 0;
        last_row = causal ? 0 : u.rows - 1;
        sub_shift = -1;
        if (!causal) sub_shift = wave_sub_shift(row_len);
        lane = threadIdx.x & 63;
#pragma unroll
        for (int f = 0; f < NF; ++f) { E[f] = 0.0f; pk[f] = 0; inv[f] = 1.0f; scale[f] = 1.0f; }
        A = 0.0f;
    }
    template <class Row>
    __device__ __forceinline__ void load_row(Row row, float (&iv)[NF], float (&sc)[NF]) const {
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            iv[f] = ri[row * NF + f];
            sc[f] = rs[row * NF + f];
        }
    }
    __device__ __forceinline__ void begin_dense(int64_t e0, int le) {
        cur.begin(e0, __builtin_amdgcn_readfirstlane(le - lane * kVec), kWG * kVec, row_len);
        cur.row = __builtin_amdgcn_readfirstlane(cur.row);
        cur.col = __builtin_amdgcn_readfirstlane(cur.col);
    }
    __device__ __forceinline__ void set_row(int64_t row) { load_row(row, inv, scale); }

    __device__ __forceinline__ void quad(uint32_t xw0, uint32_t xw1, uint32_t gw0, uint32_t gw1,
                                         const float (&iv)[NF], const float (&sc)[NF]) {
        const float xv[4] = {bf16_lo(xw0), bf16_hi(xw0), bf16_lo(xw1), bf16_hi(xw1)};
        const float gv[4] = {bf16_lo(gw0), bf16_hi(gw0), bf16_lo(gw1), bf16_hi(gw1)};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = gv[j] * xv[j];
            A = fmaf(a, a, A);
        }
        one_format<F0>(xv, gv, iv[0], sc[0], E[0], pk[0]);
        if constexpr (NF > 1) one_format<F1>(xv, gv, iv[1], sc[1], E[1], pk[1]);
    }
    __device__ __forceinline__ void vec(const u32x4& xv, const u32x4& gv, const float (&iv)[NF],
                                        const float (&sc)[NF]) {
        quad(xv.x, xv.y, gv.x, gv.y, iv, sc);
        quad(xv.z, xv.w, gv.z, gv.w, iv, sc);
    }

    template <int U>
    __device__ __forceinline__ void full(int64_t eu, int le, int64_t stride) {
        const gptr128_t bx = reinterpret_cast<gptr128_t>(x + eu);
        const gptr128_t bg = reinterpret_cast<gptr128_t>(g + eu);
        const int lv = le / kVec;
        const int64_t sv = stride / kVec;
        u32x4 xr[U], gr[U];
        if (keep_x) {
#pragma unroll
            for (int k = 0; k < U; ++k) xr[k] = load128<false>(bx + k * sv + lv);
        } else {
#pragma unroll
            for (int k = 0; k < U; ++k) xr[k] = load128<true>(bx + k * sv + lv);
        }
#pragma unroll
        for (int k = 0; k < U; ++k) gr[k] = load128<true>(bg + k * sv + lv);
        // rows of the wave's U steps
        int32_t row_a[U], rem[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            row_a[k] = cur.row;
            rem[k] = row_len - cur.col;                // elements of row_a left from the wave's first lane on
            cur.advance();
        }
        if constexpr (SHORT) {
            // short rows (8 << sub_shift elements, a divisor of 512): a step covers whole rows, the
            // lane's row is the wave's first row plus lane >> sub_shift
#pragma unroll
            for (int k = 0; k < U; ++k) {
                float iv[NF], sc[NF];
                load_row((uint32_t)(row_a[k] + (lane >> sub_shift)), iv, sc);     // = wave_lane_row
                vec(xr[k], gr[k], iv, sc);
            }
            return;
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            float iv[NF], sc[NF];
            load_row((uint32_t)row_a[k], iv, sc);      // uniform: scalar loads
            if (rem[k] >= 64 * kVec) {                 // the whole step lies in one row: scalar operands
                vec(xr[k], gr[k], iv, sc);
            } else {
                float ib[NF], sb[NF];
                load_row((uint32_t)(row_a[k] < last_row ? row_a[k] + 1 : last_row), ib, sb);
                const bool second = lane * kVec >= rem[k];
#pragma unroll
                for (int f = 0; f < NF; ++f) {
                    ib[f] = second ? ib[f] : iv[f];
                    sb[f] = second ? sb[f] : sc[f];
                }
                vec(xr[k], gr[k], ib, sb);
            }
        }
    }

    template <int U>
    __device__ __forceinline__ void full_masked(int64_t e, int stride, int count, int tail) {
        const gptr128_t px = reinterpret_cast<gptr128_t>(x + e);
        const gptr128_t pg = reinterpret_cast<gptr128_t>(g + e);
        const int sv = stride / kVec;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        u32x4 xr[U], gr[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            xr[k] = k < count ? load128<true>(px + k * sv) : zero;
            gr[k] = k < count ? load128<true>(pg + k * sv) : zero;
        }
        if (tail < kVec) {
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (k == count - 1) { xr[k] = keep_leading(xr[k], tail); gr[k] = keep_leading(gr[k], tail); }
        }
#pragma unroll
        for (int k = 0; k < U; ++k)
            if (k < count) vec(xr[k], gr[k], inv, scale);
    }

    // Not reached for the units this context is given (rows of whole vectors, aligned causal
    // rows); kept correct: the element's row by division, or the row the causal walker named.
    __device__ __forceinline__ void partial(int64_t e, int jlo, int jhi) {
        const u32x4 xv = gather8(x, e, jlo, jhi);
        const u32x4 gv = gather8(g, e, jlo, jhi);
        float iv[NF], sc[NF];
        if (!causal && row_len > 0) {
            load_row((e + jlo) / row_len, iv, sc);
        } else {
#pragma unroll
            for (int f = 0; f < NF; ++f) { iv[f] = inv[f]; sc[f] = scale[f]; }
        }
        vec(xv, gv, iv, sc);
    }
};

template <class Ctx, int NF>
__device__ __forceinline__ void sens_body(const ResolvedUnit* __restrict__ runits,
                                          const ChunkRef* __restrict__ map, uint32_t n_chunks,
                                          float* __restrict__ partials) {
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    uint32_t c = blockIdx.x;
    if (c >= n_chunks) return;
    ChunkRef ref = map[c];
    while (true) {
        const ResolvedUnit u = runits[ref.unit];
        const uint32_t local = ref.local;
        const uint32_t slot_id = ref.slot;
        const uint32_t cn = c + gridDim.x;
        const bool more = cn < n_chunks;
        if (more) ref = map[cn];                    // next chunk's entry travels while this one streams

        Ctx ctx;
        ctx.init(u);
        walk_chunk(u, local, tid, ctx);

        float v[NF + 1];
#pragma unroll
        for (int f = 0; f < NF; ++f) v[f] = wave_sum(ctx.E[f]);
        v[NF] = wave_sum(ctx.A);
        if (lane == 0) {
            float* slot = partials + ((size_t)slot_id * kWaves + wave) * (NF + 1);
#pragma unroll
            for (int k = 0; k <= NF; ++k) slot[k] = v[k];
        }
        if (!more) break;
        c = cn;
    }
}

// 7 waves per SIMD (72 VGPRs): at 8 (64 VGPRs) the compiler cannot keep a group's eight loads in
// flight and issues them one or two at a time between the arithmetic.
#ifndef AMPSENS_SENS_WAVES
#define AMPSENS_SENS_WAVES 7
#endif
template <int NF, int F0, int F1, bool POW2>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(AMPSENS_SENS_WAVES, AMPSENS_SENS_WAVES))) void sens_kernel(const ResolvedUnit* __restrict__ runits,
                                                   const ChunkRef* __restrict__ map,
                                                   uint32_t n_chunks, float* __restrict__ partials) {
    saturating_fp8_conversions();
    sens_body<SensCtx<NF, F0, F1, POW2>, NF>(runits, map, n_chunks, partials);
}

#ifndef AMPSENS_WROWS_WAVES
#define AMPSENS_WROWS_WAVES 6
#endif
template <int NF, int F0, int F1, bool SHORT>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(AMPSENS_WROWS_WAVES, AMPSENS_WROWS_WAVES))) void sens_wrows_kernel(const ResolvedUnit* __restrict__ runits,
                                                        const ChunkRef* __restrict__ map,
                                                        uint32_t n_chunks, float* __restrict__ partials) {
    saturating_fp8_conversions();
    sens_body<SensWaveRowCtx<NF, F0, F1, SHORT>, NF>(runits, map, n_chunks, partials);
}

#ifndef AMPSENS_ROWS_WAVES
#define AMPSENS_ROWS_WAVES 4
#endif
template <int NF, int F0, int F1>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(AMPSENS_ROWS_WAVES, AMPSENS_ROWS_WAVES))) void sens_rows_kernel(const ResolvedUnit* __restrict__ runits,
                                                        const ChunkRef* __restrict__ map,
                                                        uint32_t n_chunks, float* __restrict__ partials) {
    saturating_fp8_conversions();
    sens_body<SensRowCtx<NF, F0, F1>, NF>(runits, map, n_chunks, partials);
}

// ---- the weight kernel ------------------------------------------------------------------------
// A weight W is shared by the R samples of its op; only the gradient differs.  This kernel reads a
// chunk of W once for up to kWBatch samples, forms x, and x - xtilde for every format, once, and
// then streams the samples' gradient chunks against them: 7 VALU operations per element pair
// instead of 16, and W's bytes once per batch instead of once per sample.  Each thread keeps one
// 8-element vector of W per step; sums are kept per sample and written to the same per-wave
// partial slots the streaming kernel would have used, so the finalisation does not change.
// ROWS: the scales of W come from a [K][NF] table (one per output channel), followed with a
// RowCursor; they are needed once per vector of W and batch, not per sample.
template <int NF, int F0, int F1, bool ROWS>
__global__ __launch_bounds__(kWG) void sens_w_kernel(const WGroup* __restrict__ groups, uint32_t n_groups,
                                                     uint32_t n_items,
                                                     const ResolvedUnit* __restrict__ runits,
                                                     const uint32_t* __restrict__ chunk_begin,
                                                     float* __restrict__ partials) {
    saturating_fp8_conversions();
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    for (uint32_t item = blockIdx.x; item < n_items; item += gridDim.x) {
        uint32_t gi = 0, ghi = n_groups;                        // the last group whose first item is <= item
        while (ghi - gi > 1) {
            const uint32_t mid = (gi + ghi) >> 1;
            if (groups[mid].item_begin <= item) gi = mid; else ghi = mid;
        }
        const WGroup G = groups[gi];
        const uint32_t batches = (G.members + kWBatch - 1) / kWBatch;
        const uint32_t rel = item - G.item_begin;
        const uint32_t j = rel / batches;                       // chunk of W
        const uint32_t r0 = (rel % batches) * kWBatch;          // first member of the batch
        const int nb = (int)(G.members - r0 < (uint32_t)kWBatch ? G.members - r0 : (uint32_t)kWBatch);
        const ResolvedUnit u0 = runits[G.first_unit + r0 * G.unit_stride];
        gptr16_t gp[kWBatch];
        uint32_t slot[kWBatch];
#pragma unroll
        for (int k = 0; k < kWBatch; ++k) {
            const uint32_t ui = G.first_unit + (r0 + (k < nb ? k : 0)) * G.unit_stride;
            gp[k] = (gptr16_t)runits[ui].dx;
            slot[k] = chunk_begin[ui] + j;
        }
        float inv[NF], scale[NF];
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            if constexpr (ROWS) {
                inv[f] = 1.0f;                      // fetched per vector below
                scale[f] = 1.0f;
            } else {
                inv[f] = u0.inv[f];
                scale[f] = u0.scale[f];
            }
        }
        float A[kWBatch], E[NF][kWBatch];
#pragma unroll
        for (int k = 0; k < kWBatch; ++k) {
            A[k] = 0.0f;
#pragma unroll
            for (int f = 0; f < NF; ++f) E[f][k] = 0.0f;
        }
        const int64_t base = (int64_t)j * kChunkVecs * kVec;    // the unit starts on the 16-byte grid
        const gptr128_t px = reinterpret_cast<gptr128_t>((gptr16_t)u0.x + base);
        int pk = 0;
        RowCursor cur;
        if constexpr (ROWS) cur.begin(base, tid * kVec, kWG * kVec, u0.cols);
        // A full batch (the usual case) gets a copy of the loop without the per-member tests, so that
        // the compiler can wait for the gradient loads one by one instead of for all of them.
        auto steps = [&](auto full_batch) {
        constexpr bool kFull = decltype(full_batch)::value;
        const int nbe = kFull ? kWBatch : nb;
#pragma unroll 1
        for (int s = 0; s < kChunkVecs / kWG; ++s) {
            const int v = s * kWG + tid;
            const u32x4 xw = load128<false>(px + v);
            if constexpr (ROWS) {
#pragma unroll
                for (int f = 0; f < NF; ++f) {
                    inv[f] = ((gptrf_t)u0.row_inv)[(uint32_t)cur.row * NF + f];
                    scale[f] = ((gptrf_t)u0.row_scale)[(uint32_t)cur.row * NF + f];
                }
                cur.advance();
            }
            u32x4 gr[kWLoad];
#pragma unroll
            for (int k = 0; k < kWLoad; ++k)
                if (k < nbe) gr[k] = load128<true>(reinterpret_cast<gptr128_t>(gp[k] + base) + v);
            // x and the quantisation error of every format, once
            const uint32_t w4[4] = {xw.x, xw.y, xw.z, xw.w};
            float xv[kVec], ev[NF][kVec];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float x4[4] = {bf16_lo(w4[2 * h]), bf16_hi(w4[2 * h]), bf16_lo(w4[2 * h + 1]),
                                     bf16_hi(w4[2 * h + 1])};
#pragma unroll
                for (int i = 0; i < 4; ++i) xv[4 * h + i] = x4[i];
#pragma unroll
                for (int f = 0; f < NF; ++f) {
                    float q4[4];
                    if (f == 0) {
                        pk = Fp8<F0>::pack(x4[0] * inv[0], x4[1] * inv[0], pk, false);
                        pk = Fp8<F0>::pack(x4[2] * inv[0], x4[3] * inv[0], pk, true);
                        const float2_t a = Fp8<F0>::unpack(pk, false), b = Fp8<F0>::unpack(pk, true);
                        q4[0] = a.x; q4[1] = a.y; q4[2] = b.x; q4[3] = b.y;
                    } else {
                        pk = Fp8<F1>::pack(x4[0] * inv[f], x4[1] * inv[f], pk, false);
                        pk = Fp8<F1>::pack(x4[2] * inv[f], x4[3] * inv[f], pk, true);
                        const float2_t a = Fp8<F1>::unpack(pk, false), b = Fp8<F1>::unpack(pk, true);
                        q4[0] = a.x; q4[1] = a.y; q4[2] = b.x; q4[3] = b.y;
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) ev[f][4 * h + i] = fmaf(-q4[i], scale[f], x4[i]);
                }
            }
            // every sample's gradient against them, kWLoad samples in flight at a time
#pragma unroll
            for (int k0 = 0; k0 < kWBatch; k0 += kWLoad) {
#pragma unroll
                for (int kk = 0; kk < kWLoad; ++kk) {
                    const int k = k0 + kk;
                    if (k < nbe) {
                        const uint32_t g4[4] = {gr[kk].x, gr[kk].y, gr[kk].z, gr[kk].w};
                        // the slot is free: fetch the gradient of sample k + kWLoad into it
                        if (k + kWLoad < kWBatch && k + kWLoad < nbe)
                            gr[kk] = load128<true>(reinterpret_cast<gptr128_t>(gp[(k + kWLoad) % kWBatch] + base) + v);
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float g0 = bf16_lo(g4[i]), g1 = bf16_hi(g4[i]);
                            const float a0 = g0 * xv[2 * i], a1 = g1 * xv[2 * i + 1];
                            A[k] = fmaf(a0, a0, A[k]);
                            A[k] = fmaf(a1, a1, A[k]);
#pragma unroll
                            for (int f = 0; f < NF; ++f) {
                                const float t0 = g0 * ev[f][2 * i], t1 = g1 * ev[f][2 * i + 1];
                                E[f][k] = fmaf(t0, t0, E[f][k]);
                                E[f][k] = fmaf(t1, t1, E[f][k]);
                            }
                        }
                    }
                }
            }
        }
        };
        if (nb == kWBatch) steps(std::true_type{}); else steps(std::false_type{});
#pragma unroll
        for (int k = 0; k < kWBatch; ++k) {
            if (k < nb) {
                float v[NF + 1];
#pragma unroll
                for (int f = 0; f < NF; ++f) v[f] = wave_sum(E[f][k]);
                v[NF] = wave_sum(A[k]);
                if (lane == 0) {
                    float* out = partials + ((size_t)slot[k] * kWaves + wave) * (NF + 1);
#pragma unroll
                    for (int i = 0; i <= NF; ++i) out[i] = v[i];
                }
            }
        }
    }
}

// One workgroup per unit: fixed-order fp64 sum of the unit's per-wave chunk partials (thread t
// adds partials t, t + 256, ...; lanes, then waves, are combined in a fixed order).
template <int NF>
__global__ __launch_bounds__(kWG) void sens_finalize_kernel(const ResolvedUnit* __restrict__ runits,
                                                            const uint32_t* __restrict__ chunk_begin,
                                                            uint32_t n_units,
                                                            const float* __restrict__ partials,
                                                            float* __restrict__ out) {
    __shared__ double red[kWaves][NF + 1];
    const uint32_t ui = blockIdx.x;
    const size_t p0 = (size_t)chunk_begin[ui] * kWaves, p1 = (size_t)chunk_begin[ui + 1] * kWaves;
    double acc[NF + 1];
#pragma unroll
    for (int k = 0; k <= NF; ++k) acc[k] = 0.0;
    for (size_t p = p0 + threadIdx.x; p < p1; p += kWG) {
#pragma unroll
        for (int k = 0; k <= NF; ++k) acc[k] += (double)partials[p * (NF + 1) + k];
    }
#pragma unroll
    for (int k = 0; k <= NF; ++k) acc[k] = wave_sum(acc[k]);
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int k = 0; k <= NF; ++k) red[threadIdx.x >> 6][k] = acc[k];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot[NF + 1];
#pragma unroll
        for (int k = 0; k <= NF; ++k) tot[k] = (red[0][k] + red[1][k]) + (red[2][k] + red[3][k]);
        const uint32_t o = runits[ui].out;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            out[o + 4 * f] = (float)tot[f];
            out[o + 4 * f + 1] = (float)tot[NF];
        }
    }
}

// ---- absmax ---------------------------------------------------------------------------------

typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

struct AbsmaxCtx {
    static constexpr bool kRollDense = false;
    gptr16_t x;
    uint32_t m;                                     // two running maxima of (bits & 0x7FFF), one per half

    // both elements of a word at once: clear the signs, packed 16-bit maximum
    __device__ __forceinline__ void word(uint32_t w) {
        const u16x2 a = __builtin_bit_cast(u16x2, m), b = __builtin_bit_cast(u16x2, w & 0x7FFF7FFFu);
        m = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
    }
    __device__ __forceinline__ uint32_t result() const {
        const uint32_t lo = m & 0xFFFFu, hi = m >> 16;
        return lo > hi ? lo : hi;
    }
    __device__ __forceinline__ void vec(const u32x4& v) { word(v.x); word(v.y); word(v.z); word(v.w); }
    __device__ __forceinline__ void begin_dense(int64_t, int) {}
    __device__ __forceinline__ void set_row(int64_t) {}

    template <int U>
    __device__ __forceinline__ void full(int64_t eu, int le, int64_t stride) {
        const gptr128_t bx = reinterpret_cast<gptr128_t>(x + eu);
        const int lv = le / kVec;
        const int64_t sv = stride / kVec;
        u32x4 xr[U];
#pragma unroll
        for (int k = 0; k < U; ++k) xr[k] = load128<true>(bx + k * sv + lv);
#pragma unroll
        for (int k = 0; k < U; ++k) vec(xr[k]);
    }
    template <int U>
    __device__ __forceinline__ void full_masked(int64_t e, int stride, int count, int tail) {
        const gptr128_t px = reinterpret_cast<gptr128_t>(x + e);
        const int sv = stride / kVec;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        u32x4 xr[U];
#pragma unroll
        for (int k = 0; k < U; ++k) xr[k] = k < count ? load128<true>(px + k * sv) : zero;
        if (tail < kVec) {
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (k == count - 1) xr[k] = keep_leading(xr[k], tail);
        }
#pragma unroll
        for (int k = 0; k < U; ++k) vec(xr[k]);
    }
    __device__ __forceinline__ void partial(int64_t e, int jlo, int jhi) { vec(gather8(x, e, jlo, jhi)); }
};

#ifndef AMPSENS_ABSMAX_WAVES
#define AMPSENS_ABSMAX_WAVES 8
#endif
// Per-wave maxima of every chunk go to their own slots: integer max is exact and order-free,
// and without atomics there is no contention on the few per-tensor words.
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(AMPSENS_ABSMAX_WAVES, AMPSENS_ABSMAX_WAVES))) void absmax_kernel(const ResolvedUnit* __restrict__ runits,
                                                     const ChunkRef* __restrict__ map,
                                                     uint32_t n_chunks,
                                                     uint32_t* __restrict__ partial_max) {
    const int tid = threadIdx.x;
    uint32_t c = blockIdx.x;
    if (c >= n_chunks) return;
    ChunkRef ref = map[c];
    while (true) {
        const ResolvedUnit u = runits[ref.unit];
        const uint32_t local = ref.local;
        const uint32_t slot_id = ref.slot;
        const uint32_t cn = c + gridDim.x;
        const bool more = cn < n_chunks;
        if (more) ref = map[cn];
        AbsmaxCtx ctx;
        ctx.x = (gptr16_t)u.x;
        ctx.m = 0;
        walk_chunk(u, local, tid, ctx);
        const uint32_t m = wave_max(ctx.result());
        if ((tid & 63) == 0) partial_max[(size_t)slot_id * kWaves + (tid >> 6)] = m;
        if (!more) break;
        c = cn;
    }
}

__device__ __forceinline__ float fmax_of(int fmt) { return fmt == 0 ? 448.0f : 57344.0f; }

// amax (as the maximum of bits & 0x7FFF) -> amax and the scales of every format.  A format code
// with kScalePow2 set asks for the smallest power of two s with amax / s <= FMAX and inv = 1 / s
// (both exact) instead of amax / FMAX and FMAX / amax.
constexpr int kScalePow2 = 0x100;
__device__ __forceinline__ void write_scales(uint32_t bits, int n_fmts, int fmt0, int fmt1, float* amax_out,
                                             float* scale_out, float* inv_out) {
    const float amax = __uint_as_float(bits << 16);
    *amax_out = amax;
    for (int f = 0; f < n_fmts; ++f) {
        const int code = f == 0 ? fmt0 : fmt1;
        const float fm = fmax_of(code & 0xFF);
        float scale = 1.0f, inv = 1.0f;
        if (code & kScalePow2) {
            // FMAX = 1.75 * 2^eF; amax = m * 2^e with m in [1, 2): k = e - eF, one more if m > 1.75
            const int e_field = (int)(bits >> 7) & 0xFF;                // bf16 exponent field
            if (e_field != 0 && e_field != 0xFF) {
                const int k = e_field - 127 - ((code & 0xFF) == 0 ? 8 : 15) + ((bits & 0x7Fu) > 96u ? 1 : 0);
                if (k >= -127 && k <= 127) {
                    scale = k >= -126 ? __uint_as_float((uint32_t)(k + 127) << 23)
                                      : __uint_as_float(1u << (k + 149));
                    inv = __uint_as_float((uint32_t)(127 - k) << 23);
                }
            }
        } else if (amax != 0.0f) {
            scale = amax / fm;                      // correctly rounded fp32 divisions
            inv = fm / amax;
            if (__builtin_isinf(inv)) { scale = 1.0f; inv = 1.0f; }
        }
        scale_out[f] = scale;
        inv_out[f] = inv;
    }
}

// One workgroup of 1024 threads per tensor (unit t of an absmax call is tensor t).
constexpr int kFinThreads = 1024;
__global__ __launch_bounds__(kFinThreads) void absmax_finalize_kernel(const uint32_t* __restrict__ chunk_begin,
                                                              const uint32_t* __restrict__ partial_max,
                                                              int n_fmts, int fmt0, int fmt1,
                                                              float* __restrict__ amax_out,
                                                              float* __restrict__ scale_out,
                                                              float* __restrict__ inv_out,
                                                              uint32_t* __restrict__ flags_out) {
    __shared__ uint32_t red[kFinThreads / 64];
    const int t = blockIdx.x;
    const size_t p0 = (size_t)chunk_begin[t] * kWaves, p1 = (size_t)chunk_begin[t + 1] * kWaves;
    uint32_t m = 0;
#pragma unroll 4
    for (size_t p = p0 + threadIdx.x; p < p1; p += kFinThreads) {
        const uint32_t v = partial_max[p];
        m = m > v ? m : v;
    }
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x != 0) return;
    uint32_t bits = 0;
    for (int w = 0; w < kFinThreads / 64; ++w) bits = bits > red[w] ? bits : red[w];
    flags_out[t] = bits >= 0x7F80u ? 1u : 0u;
    write_scales(bits, n_fmts, fmt0, fmt1, &amax_out[t], &scale_out[t * n_fmts], &inv_out[t * n_fmts]);
}

// ---- absmax and scales per row ----------------------------------------------------------------
// A wave owns a run of consecutive rows of one tensor.  Rows made of whole, aligned vectors are
// read with 128-bit loads by a group of lanes sized so that every lane has about four vectors to
// fetch (a 128-element row: 4 lanes, 16 rows per wave step); other rows are read element by
// element by the whole wave.  Every row is reduced inside its lane group and written by one lane:
// no partials, no second kernel.  flags must be zero before the launch.
__device__ __forceinline__ uint32_t max_words(uint32_t m, const u32x4& v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t lo = w[k] & 0x7FFFu, hi = (w[k] >> 16) & 0x7FFFu;
        m = m > lo ? m : lo;
        m = m > hi ? m : hi;
    }
    return m;
}

__global__ __launch_bounds__(kWG) void zero_u32_kernel(uint32_t* __restrict__ p, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

__global__ __launch_bounds__(kWG) void absmax_rows_kernel(const RowTensor* __restrict__ tensors,
                                                          uint32_t n_tensors, uint32_t n_items,
                                                          int n_fmts, int fmt0, int fmt1,
                                                          float* __restrict__ amax_out,
                                                          float* __restrict__ scale_out,
                                                          float* __restrict__ inv_out,
                                                          uint32_t* __restrict__ flags_out) {
    const int lane = threadIdx.x & 63;
    const uint32_t n_waves = gridDim.x * kWaves;
    for (uint32_t item = blockIdx.x * kWaves + (threadIdx.x >> 6); item < n_items; item += n_waves) {
        uint32_t lo = 0, hi = n_tensors;            // the last tensor whose first item is <= item
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (tensors[mid].item_begin <= item) lo = mid; else hi = mid;
        }
        const RowTensor T = tensors[lo];
        const int L = T.aligned ? absmax_row_lanes(T.row_len, T.causal_rows > 0) : 64;   // lanes per row
        const int G = 64 / L, sub = lane / L, sl = lane - sub * L;
        // rows [row0, row1) of the tensor; i0 = index of row0 inside its matrix (causal)
        auto run = [&](int64_t row0, int64_t row1, int32_t i0) {
            for (int64_t rb = row0; rb < row1; rb += G) {
                const int64_t rho = rb + sub;
                const bool live = rho < row1;
                int32_t len = T.row_len;
                if (T.causal_rows > 0) {
                    const int32_t i = (int32_t)(((int64_t)i0 + (rho - row0)) % T.causal_rows);
                    int64_t l = (int64_t)i + 1 + ((int64_t)T.row_len - T.causal_rows);
                    len = (int32_t)(l < 0 ? 0 : (l > T.row_len ? T.row_len : l));
                }
                uint32_t m = 0;
                if (live && T.aligned) {
                    const int nvr = (len + kVec - 1) / kVec;
                    const int tail = len - (nvr - 1) * kVec;
                    const gptr128_t p = reinterpret_cast<gptr128_t>((gptr16_t)T.x + rho * T.row_len);
                    const int nwhole = tail < kVec ? nvr - 1 : nvr;   // vectors that need no masking
                    int v = sl;
                    for (; v + 3 * L < nwhole; v += 4 * L) {       // four whole vectors in flight
                        const u32x4 a = load128<true>(p + v), b = load128<true>(p + v + L);
                        const u32x4 c = load128<true>(p + v + 2 * L), d = load128<true>(p + v + 3 * L);
                        m = max_words(max_words(max_words(max_words(m, a), b), c), d);
                    }
                    for (; v < nvr; v += L) {
                        u32x4 a = load128<true>(p + v);
                        if (v == nvr - 1 && tail < kVec) a = keep_leading(a, tail);
                        m = max_words(m, a);
                    }
                } else if (live) {
                    const gptr16_t p = (gptr16_t)T.x + rho * T.row_len;
                    for (int32_t j = sl; j < len; j += L) {
                        const uint32_t h = (uint32_t)p[j] & 0x7FFFu;
                        m = m > h ? m : h;
                    }
                }
                for (int o = 1; o < L; o <<= 1) {              // L is the same for the whole wave
                    const uint32_t w = (uint32_t)__shfl_xor((int)m, o);
                    m = m > w ? m : w;
                }
                if (live && sl == 0) {
                    const int64_t o = (int64_t)T.out_row + rho;
                    write_scales(m, n_fmts, fmt0, fmt1, &amax_out[o], &scale_out[o * n_fmts], &inv_out[o * n_fmts]);
                    if (m >= 0x7F80u) atomicOr(&flags_out[lo], 1u);
                }
            }
        };
        const uint32_t rel = item - T.item_begin;
        if (T.items_per_mat > 0) {
            const int64_t mat = rel / T.items_per_mat;
            const int32_t slot = (int32_t)(rel % T.items_per_mat);
            const int32_t mirror = (T.causal_rows + kBandRows - 1) / kBandRows - 1 - slot;
            const int64_t base = mat * T.causal_rows;
            const int32_t a0 = slot * kBandRows, b0 = mirror * kBandRows;
            run(base + a0, base + (a0 + kBandRows < T.causal_rows ? a0 + kBandRows : T.causal_rows), a0);
            if (mirror > slot)
                run(base + b0, base + (b0 + kBandRows < T.causal_rows ? b0 + kBandRows : T.causal_rows), b0);
        } else {
            const int64_t row0 = (int64_t)rel * T.rows_per_item;
            run(row0, row0 + T.rows_per_item < T.n_rows ? row0 + T.rows_per_item : T.n_rows, 0);
        }
    }
}

// ---- the single-read pass for operands with one scale per row ------------------------------------
// The row-scaled pass without a separate absmax pass: a workgroup takes a tile of rows, `lanes`
// threads per row; every thread loads its vectors of the row once, folds them into the row's absmax
// and parks them in LDS (its own slots, so no barrier guards them); the absmax is reduced over the
// row's threads (cross-lane moves inside a wave, LDS and one barrier when a row spans several waves),
// the scales of every format are derived with the arithmetic of write_scales and written to the
// operand's tables by one thread per row, and the row's gradient is streamed against the parked
// vectors.  Geometry: FusedGeom in `head`; causal units choose the lanes tile by tile (internal.h).

// One of the four numbers write_scales derives from a row's amax: scale (want_inv false) or
// reciprocal (true) of format `code` (which may carry kScalePow2).  Same results bit for bit; the
// case "the reciprocal overflows fp32, so both are 1" is decided from amax alone: FMAX / amax rounds
// to infinity exactly for amax <= 1.75 * 2^-120 (E4M3, bits 0x03E0) and 1.75 * 2^-113 (E5M2, 0x0760).
__device__ __forceinline__ float scale_quantity(uint32_t bits, int code, bool want_inv) {
    const int fmt = code & 0xFF;
    if (code & kScalePow2) {
        const int e_field = (int)(bits >> 7) & 0xFF;
        if (e_field == 0 || e_field == 0xFF) return 1.0f;
        const int k = e_field - 127 - (fmt == 0 ? 8 : 15) + ((bits & 0x7Fu) > 96u ? 1 : 0);
        if (k < -127 || k > 127) return 1.0f;
        if (want_inv) return __uint_as_float((uint32_t)(127 - k) << 23);
        return k >= -126 ? __uint_as_float((uint32_t)(k + 127) << 23) : __uint_as_float(1u << (k + 149));
    }
    if (bits <= (fmt == 0 ? 0x03E0u : 0x0760u)) return 1.0f;     // amax == 0, or the reciprocal would be infinite
    const float amax = __uint_as_float(bits << 16);
    const float fm = fmax_of(fmt);
    return want_inv ? fm / amax : amax / fm;
}

// The two divisions of scale_quantity, looked up.  amax = a * 2^(e-127) with a = 1 + m/128 one of 128 values:
// table[(f * 2 + inv) * 128 + m] holds a / FMAX_f (inv = 0) or FMAX_f / a (inv = 1), computed by the same fp32
// divisions, and scaling by a power of two commutes with a correctly rounded division as long as the result
// is a normal number: amax / FMAX = table * 2^(e-127), FMAX / amax = table * 2^(127-e), bit for bit.  Exponent
// fields below 20 (results that can be subnormal, the reciprocal-overflow rule) and 255 take the divisions.
// The four numbers of a mantissa are neighbours, so the four threads of a quad, which ask for the four numbers
// of one row, read four consecutive words (no bank conflict inside the quad).
constexpr int kScaleTableWords = 128 * 4;
__device__ __forceinline__ void fill_scale_table(float* table, int code0, int code1) {
    for (int i = threadIdx.x; i < kScaleTableWords; i += kWG) {
        const int which = i & 3;                               // format * 2 + reciprocal
        const float fm = fmax_of(((which >> 1) == 0 ? code0 : code1) & 0xFF);
        const float a = __uint_as_float(0x3F800000u | ((uint32_t)(i >> 2) << 16));
        table[i] = (which & 1) ? fm / a : a / fm;
    }
}
__device__ __forceinline__ float scale_quantity(uint32_t bits, int f, int code, bool want_inv, const float* table) {
    const int e = (int)(bits >> 7);
    if ((code & kScalePow2) || e < 20 || e >= 255) return scale_quantity(bits, code, want_inv);
    const float t = table[((int)(bits & 127u) << 2) | (f * 2 + (want_inv ? 1 : 0))];
    return __builtin_ldexpf(t, want_inv ? 127 - e : e - 127);
}

// max(v, v of the lane a DPP pattern names); every lane has a source in the patterns used here
template <int CTRL>
__device__ __forceinline__ uint32_t max_with_dpp(uint32_t v) {
    const uint32_t w = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
    return w > v ? w : v;
}

template <int CTRL>
__device__ __forceinline__ float quad_broadcast(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// The row tiles of one chunk, in the order a workgroup takes them.  Uniform over the workgroup
// except for live / row / len.
struct FusedTile {
    bool valid;                                    // there is such a tile
    int lanes_log2;                                // threads per row
    int nv_exact;                                  // vectors k < nv_exact of every thread are whole vectors of a live row
    int nv;                                        // vectors per thread (whole groups); those past a row's end are masked
    bool live;                                     // this thread's row exists
    int64_t row;                                   // row of the unit (table index); the tile's first row when not live
    int32_t len;                                   // valid elements of the row
    int64_t row0;                                  // the tile's first row (thread t holds row0 + (t >> lanes_log2)): the same for the workgroup
};
struct FusedTileWalk {
    int32_t rows, cols;
    bool causal;
    FusedGeom geo;
    int tid;
    int64_t next_tile;                             // dense: tile of the unit; causal: tile of the matrix
    int left;                                      // tiles still to come
    int64_t mat_row0;                              // causal: first row of the matrix in the unit

    __device__ __forceinline__ void begin(const ResolvedUnit& u, const FusedGeom& g, uint32_t local, int tid_) {
        rows = u.rows; cols = u.cols; geo = g; tid = tid_;
        causal = (u.flags & kUnitCausal) != 0;
        left = g.tiles;
        if (!causal) {
            next_tile = (int64_t)local * g.tiles;
            mat_row0 = 0;
        } else {
            const uint32_t mat = local / u.chunks_per_mat;
            mat_row0 = (int64_t)mat * rows;
            next_tile = (int64_t)(local % u.chunks_per_mat) * g.tiles;
        }
    }
    static __device__ __forceinline__ int whole_groups_down(int v) { return v / kFusedGroup * kFusedGroup; }
    static __device__ __forceinline__ int whole_groups_up(int v) { return (v + kFusedGroup - 1) / kFusedGroup * kFusedGroup; }
    __device__ __forceinline__ FusedTile next() {
        FusedTile t;
        t.valid = false; t.lanes_log2 = 2; t.nv_exact = 0; t.nv = 0; t.live = false; t.row = 0; t.len = 0; t.row0 = 0;
        if (left <= 0) return t;
        --left;
        if (!causal) {
            const int lg = geo.lanes_log2;
            const int RT = kWG >> lg;
            const int64_t r0 = next_tile * RT;
            if (r0 >= rows) { left = 0; return t; }
            ++next_tile;
            const int64_t r = r0 + (tid >> lg);
            const int32_t row_vecs = cols / kVec;
            t.valid = true;
            t.lanes_log2 = lg;
            t.live = r < rows;
            t.row = t.live ? r : r0;
            t.row0 = r0;
            t.len = cols;
            t.nv = geo.nv;
            t.nv_exact = r0 + RT <= rows ? whole_groups_down(row_vecs >> lg) : 0;
            return t;
        }
        FusedCausalTile ct;
        if (!fused_causal_tile(rows, cols, next_tile, &ct)) { left = 0; return t; }
        ++next_tile;
        const int lg = ct.lanes_log2;
        const int RT = kWG >> lg;
        const int32_t i = (int32_t)ct.row0 + (tid >> lg);
        t.valid = true;
        t.lanes_log2 = lg;
        t.live = (tid >> lg) < ct.n_rows;
        t.row = mat_row0 + (t.live ? i : (int32_t)ct.row0);
        t.row0 = mat_row0 + (int32_t)ct.row0;
        t.len = t.live ? causal_row_len(i, rows, cols) : 0;
        const int32_t len_min = causal_row_len((int32_t)ct.row0, rows, cols);
        const int32_t len_max = causal_row_len((int32_t)ct.row0 + ct.n_rows - 1, rows, cols);
        const int32_t vec_max = (len_max + kVec - 1) / kVec;
        t.nv = whole_groups_up((vec_max + (1 << lg) - 1) >> lg);
        t.nv_exact = ct.n_rows == RT ? whole_groups_down((len_min / kVec) >> lg) : 0;
        return t;
    }
};

template <int NF, int F0, int F1, bool POW2>
struct FusedRows {
    static constexpr int kG = kFusedGroup;         // vectors of x (and of the gradient) in flight per thread
    gptr16_t x, g;
    float* ts;                                     // scale[row][NF]
    float* ti;                                     // inv[row][NF]
    int32_t cols;
    int code0, code1;
    float E[NF], A;
    int pk[NF];
    uint32_t* red;                                 // LDS, [2][kWaves]: wave maxima of rows that span waves
    const float* scale_table;                      // LDS, fill_scale_table
    u32x4* stage;                                  // LDS, [nv][kWG]: this workgroup's vectors of x
    int parity;

    // POW2: iv holds the scales the codes are taken back with and mul their multiplier (one_format_pow2)
    __device__ __forceinline__ void quad(uint32_t xw0, uint32_t xw1, uint32_t gw0, uint32_t gw1,
                                         const float (&iv)[NF], const float (&sc)[NF], float mul) {
        const float xv[4] = {bf16_lo(xw0), bf16_hi(xw0), bf16_lo(xw1), bf16_hi(xw1)};
        const float gv[4] = {bf16_lo(gw0), bf16_hi(gw0), bf16_lo(gw1), bf16_hi(gw1)};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float a = gv[q] * xv[q];
            A = fmaf(a, a, A);
        }
        if constexpr (POW2) {                          // scales of the power-of-two rule, derived from this very row
            one_format_pow2<F0>(xw0, xw1, xv, gv, sc[0], iv[0], mul, E[0], pk[0]);
            if constexpr (NF > 1) one_format_pow2<F1>(xw0, xw1, xv, gv, sc[1], iv[1], mul, E[1], pk[1]);
        } else {
            one_format<F0>(xv, gv, iv[0], sc[0], E[0], pk[0]);
            if constexpr (NF > 1) one_format<F1>(xv, gv, iv[1], sc[1], E[1], pk[1]);
        }
    }

    // From the packed maxima a thread folded over its vectors of a row (m2) to the row's scales: the
    // maximum over the row's threads, the scales by the call's rule (each thread of a quad derives one of
    // the four numbers), the row's entries of the tables.  POW2: iv returns the scales the codes are
    // taken back with and mul their multiplier (one_format_pow2).
    __device__ __forceinline__ void row_scales(const FusedTile& t, uint32_t m2, float (&sc)[NF], float (&iv)[NF], float& mul) {
        const uint32_t m = row_max(m2, t.lanes_log2);
        scales_of_row(m, t.live && (threadIdx.x & ((1 << t.lanes_log2) - 1)) == 0, ts, ti, t.row, sc, iv, mul);
    }

    // Maximum over the 2^lg threads of a row (consecutive lanes, lg >= 2): quads, then halves of a 16-lane
    // row, then its mirror image, by DPP; the steps across 16-lane rows by lane shuffles; rows that span
    // waves (lg > 6, uniform over the workgroup) through LDS and one barrier.
    __device__ __forceinline__ uint32_t row_max(uint32_t m2, int lg) {
        const int tid = threadIdx.x;
        uint32_t m = (m2 & 0xFFFFu) > (m2 >> 16) ? (m2 & 0xFFFFu) : (m2 >> 16);
        m = max_with_dpp<0xB1>(m);                                 // quad_perm [1, 0, 3, 2]
        m = max_with_dpp<0x4E>(m);                                 // quad_perm [2, 3, 0, 1]
        if (lg > 2) m = max_with_dpp<0x141>(m);                    // row_half_mirror
        if (lg > 3) m = max_with_dpp<0x140>(m);                    // row_mirror
        if (lg > 4) {
            const uint32_t w = (uint32_t)__shfl_xor((int)m, 16);
            m = w > m ? w : m;
        }
        if (lg > 5) {
            const uint32_t w = (uint32_t)__shfl_xor((int)m, 32);
            m = w > m ? w : m;
        }
        if (lg > 6) {                                  // the row spans 2 or 4 waves (uniform over the workgroup)
            const int wave = tid >> 6;
            if ((tid & 63) == 0) red[parity * kWaves + wave] = m;
            __syncthreads();
            const int w0 = lg == 7 ? (wave & 2) : 0, wn = lg == 7 ? 2 : 4;
            for (int w = 0; w < wn; ++w) {
                const uint32_t v = red[parity * kWaves + w0 + w];
                m = m > v ? m : v;
            }
            parity ^= 1;
        }
        return m;
    }

    // The scales of the row whose absmax (as bits) is m: each thread of a quad derives one of (scale_0, inv_0,
    // scale_1, inv_1), then the quad shares them; the thread with `writer` set stores the row's table entries.
    __device__ __forceinline__ void scales_of_row(uint32_t m, bool writer, float* ts_base, float* ti_base, int64_t row,
                                                  float (&sc)[NF], float (&iv)[NF], float& mul) {
        {
            const int q = threadIdx.x & 3;
            const int f = NF > 1 ? (q >> 1) : 0;
            const float mine = scale_quantity(m, f, f == 0 ? code0 : code1, (q & 1) != 0, scale_table);
            sc[0] = quad_broadcast<0x00>(mine);
            iv[0] = quad_broadcast<0x55>(mine);
            if constexpr (NF > 1) {
                sc[1] = quad_broadcast<0xAA>(mine);
                iv[1] = quad_broadcast<0xFF>(mine);
            }
        }
        if (writer) {
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                ts_base[row * NF + f] = sc[f];
                ti_base[row * NF + f] = iv[f];
            }
        }
        mul = -1.0f;
        if constexpr (POW2) {
            // a row whose absmax is at least 1 has scales of at least 2^-15 in either format: a quarter of
            // them is a normal number; any other row is far from the overflow the quarter is for
            const bool roomy = m >= 0x3F80u;
            mul = roomy ? -4.0f : -1.0f;
#pragma unroll
            for (int f = 0; f < NF; ++f) iv[f] = roomy ? sc[f] * 0.25f : sc[f];
        }
    }

    // Tiles whose threads hold at most kFusedRegNv vectors of their row stay in registers (no LDS): the
    // vectors of x and of the gradient are all requested at once (regs_issue), and later (regs_finish) x
    // is folded into the row's absmax, the scales are derived, and the sums formed from the registers.
    // (Requesting the next tile's vectors before finishing the current one was measured and gave nothing:
    // the pass is bound by vector-instruction issue, not by exposed latency.)  Addresses and masks as in tile().
    struct Regs { u32x4 x[kFusedRegNv], g[kFusedRegNv]; };

    __device__ __forceinline__ void regs_issue(const FusedTile& t, Regs& r) {
        constexpr int NV = kFusedRegNv;
        const int lg = t.lanes_log2;
        const int j = threadIdx.x & ((1 << lg) - 1);
        if (t.nv_exact >= NV) {                        // every vector of every thread is a whole vector of a live row
            // (a tile of a dense unit, or the one-row tile of a causal row that is as long as the tile).  One base
            // for the workgroup, the tile's first row, and a 32-bit byte offset per lane that does not change
            // from tile to tile
            const gptr8_t bx = reinterpret_cast<gptr8_t>(x + t.row0 * (int64_t)cols);
            const gptr8_t bg = reinterpret_cast<gptr8_t>(g + t.row0 * (int64_t)cols);
            const uint32_t off = ((uint32_t)(threadIdx.x >> lg) * (uint32_t)cols + (uint32_t)j * kVec) * 2u;
            const uint32_t step = (uint32_t)(kVec * 2) << lg;
#pragma unroll
            for (int k = 0; k < NV; ++k) r.x[k] = load128<true>(reinterpret_cast<gptr128_t>(bx + (off + (uint32_t)k * step)));
#pragma unroll
            for (int k = 0; k < NV; ++k) r.g[k] = load128<true>(reinterpret_cast<gptr128_t>(bg + (off + (uint32_t)k * step)));
        } else {
            // vectors past a row's end are fetched from its last vector and masked later; a thread without a
            // row takes the tile's first.  The same base and 32-bit offsets (a tile spans at most 256 rows of at
            // most 8 192 elements)
            const gptr8_t bx = reinterpret_cast<gptr8_t>(x + t.row0 * (int64_t)cols);
            const gptr8_t bg = reinterpret_cast<gptr8_t>(g + t.row0 * (int64_t)cols);
            const uint32_t row_off = (uint32_t)(t.row - t.row0) * (uint32_t)cols * 2u;
            const int nvr = (t.len + kVec - 1) / kVec;
            const int last = nvr > 0 ? nvr - 1 : 0;
            uint32_t at[NV];
#pragma unroll
            for (int k = 0; k < NV; ++k) {
                const int v = j + (k << lg);
                at[k] = row_off + (uint32_t)(v < last ? v : last) * (uint32_t)(kVec * 2);
            }
#pragma unroll
            for (int k = 0; k < NV; ++k) r.x[k] = load128<true>(reinterpret_cast<gptr128_t>(bx + at[k]));
#pragma unroll
            for (int k = 0; k < NV; ++k) r.g[k] = load128<true>(reinterpret_cast<gptr128_t>(bg + at[k]));
        }
    }

    __device__ __forceinline__ void regs_finish(const FusedTile& t, Regs& r) {
        constexpr int NV = kFusedRegNv;
        const int lg = t.lanes_log2;
        const int j = threadIdx.x & ((1 << lg) - 1);
        if (t.nv_exact < NV) {
            const int32_t len = t.live ? t.len : 0;
#pragma unroll
            for (int k = 0; k < NV; ++k) {
                int c = len - (j + (k << lg)) * kVec;
                c = c < 0 ? 0 : (c > kVec ? kVec : c);
                if (__builtin_amdgcn_ballot_w64(c != kVec) != 0) {   // most waves hold whole vectors only
                    r.x[k] = keep_leading(r.x[k], c);
                    r.g[k] = keep_leading(r.g[k], c);
                }
            }
        }
        uint32_t m2 = 0;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const uint32_t w[4] = {r.x[k].x, r.x[k].y, r.x[k].z, r.x[k].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u16x2 a = __builtin_bit_cast(u16x2, m2), b = __builtin_bit_cast(u16x2, w[q] & 0x7FFF7FFFu);
                m2 = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
            }
        }
        float sc[NF], iv[NF], mul;
        row_scales(t, m2, sc, iv, mul);
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            quad(r.x[k].x, r.x[k].y, r.g[k].x, r.g[k].y, iv, sc, mul);
            quad(r.x[k].z, r.x[k].w, r.g[k].z, r.g[k].w, iv, sc, mul);
        }
    }

    // Short dense rows of 2^p vectors (p = 2 .. 4: 32 to 128 elements).  With a few threads per row every
    // load instruction of tile() touches many separate 64-byte pieces; here a tile is 1024 consecutive
    // vectors of the unit and thread t takes vectors t, t + 256, t + 512, t + 768 of it, so that every load
    // instruction of a wave reads 1 KiB of consecutive memory.  A thread's four vectors then lie in four
    // different rows; the 2^p lanes that hold a row reduce its absmax and derive its scales, vector by vector.
    __device__ __forceinline__ void wide_tile(int64_t v0, int64_t total, int p) {
        constexpr int NV = kFusedRegNv;
        const int tid = threadIdx.x;
        const gptr128_t px = reinterpret_cast<gptr128_t>(x) + v0;
        const gptr128_t pg = reinterpret_cast<gptr128_t>(g) + v0;
        u32x4 xr[NV], gr[NV];
        const bool whole = v0 + (int64_t)NV * kWG <= total;        // uniform
        const int left = whole ? NV * kWG : (int)(total - v0);     // vectors of the tile that exist (>= 1)
        const int64_t row0 = v0 >> p;                              // uniform
        if (whole) {
#pragma unroll
            for (int k = 0; k < NV; ++k) xr[k] = load128<true>(px + (tid + k * kWG));
#pragma unroll
            for (int k = 0; k < NV; ++k) gr[k] = load128<true>(pg + (tid + k * kWG));
        } else {
            int at[NV];
#pragma unroll
            for (int k = 0; k < NV; ++k) at[k] = tid + k * kWG < left ? tid + k * kWG : left - 1;
#pragma unroll
            for (int k = 0; k < NV; ++k) xr[k] = load128<true>(px + at[k]);
#pragma unroll
            for (int k = 0; k < NV; ++k) gr[k] = load128<true>(pg + at[k]);
            const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int k = 0; k < NV; ++k)
                if (tid + k * kWG >= left) { xr[k] = zero; gr[k] = zero; }
        }
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            uint32_t m2 = 0;
            const uint32_t w[4] = {xr[k].x, xr[k].y, xr[k].z, xr[k].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u16x2 a = __builtin_bit_cast(u16x2, m2), b = __builtin_bit_cast(u16x2, w[q] & 0x7FFF7FFFu);
                m2 = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
            }
            const uint32_t m = row_max(m2, p);
            // the row's table entry: the tile's first row (uniform, 64 bits) + this vector's row inside the tile
            const int in_tile = tid + k * kWG;
            const bool writer = (tid & ((1 << p) - 1)) == 0 && (whole || in_tile < left);
            float sc[NF], iv[NF], mul;
            scales_of_row(m, writer, ts + row0 * NF, ti + row0 * NF, in_tile >> p, sc, iv, mul);
            quad(xr[k].x, xr[k].y, gr[k].x, gr[k].y, iv, sc, mul);
            quad(xr[k].z, xr[k].w, gr[k].z, gr[k].w, iv, sc, mul);
        }
    }

    // One tile.  First visit: every thread loads its vectors of its row (each byte of x leaves HBM
    // here, once), folds them into the row's absmax and parks them in its own LDS slots; the absmax is
    // reduced over the row's threads and the scales derived and written to the tables.  Second visit:
    // the thread takes its vectors back from LDS and streams the gradient against them.  Loads are
    // unconditional (a thread whose vector lies past the row's end re-reads the row's last vector,
    // a thread without a row the tile's first); groups k >= nv_exact clear what does not belong to the
    // row with per-vector masks, without branches.
    __device__ __forceinline__ void tile(const FusedTile& t) {
        const int lg = t.lanes_log2;
        const int L = 1 << lg;
        const int tid = threadIdx.x;
        const int j = tid & (L - 1);
        const int nvr = (t.len + kVec - 1) / kVec;
        const int last = nvr > 0 ? nvr - 1 : 0;
        const int32_t len = t.live ? t.len : 0;
        const gptr128_t px = reinterpret_cast<gptr128_t>(x + t.row * (int64_t)cols);
        const gptr128_t pg = reinterpret_cast<gptr128_t>(g + t.row * (int64_t)cols);
        auto clamped = [&](int k) {
            const int v = j + (k << lg);
            return v < last ? v : last;
        };
        auto count = [&](int k) {                                  // elements of vector k that belong to the row
            const int c = len - (j + (k << lg)) * kVec;
            return c < 0 ? 0 : (c > kVec ? kVec : c);
        };
        auto fold = [](uint32_t m2, const u32x4& v) {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const u16x2 a = __builtin_bit_cast(u16x2, m2), b = __builtin_bit_cast(u16x2, w[q] & 0x7FFF7FFFu);
                m2 = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
            }
            return m2;
        };
        // first visit
        uint32_t m2 = 0;
        int k0 = 0;
#pragma unroll 1
        for (; k0 < t.nv_exact; k0 += kG) {
            u32x4 xr[kG];
#pragma unroll
            for (int k = 0; k < kG; ++k) xr[k] = load128<true>(px + (j + ((k0 + k) << lg)));
#pragma unroll
            for (int k = 0; k < kG; ++k) {
                m2 = fold(m2, xr[k]);
                stage[(k0 + k) * kWG + tid] = xr[k];
            }
        }
#pragma unroll 1
        for (; k0 < t.nv; k0 += kG) {
            u32x4 xr[kG];
#pragma unroll
            for (int k = 0; k < kG; ++k) xr[k] = load128<true>(px + clamped(k0 + k));
#pragma unroll
            for (int k = 0; k < kG; ++k) {
                const int c = count(k0 + k);                       // most waves hold whole vectors only: no masks then
                if (__builtin_amdgcn_ballot_w64(c != kVec) != 0) xr[k] = keep_leading(xr[k], c);
                m2 = fold(m2, xr[k]);
                stage[(k0 + k) * kWG + tid] = xr[k];
            }
        }
        float sc[NF], iv[NF], mul;
        row_scales(t, m2, sc, iv, mul);
        // second visit: x from this thread's LDS slots (already cleared where it had to be), the gradient from
        // HBM.  Vectors outside the row are (0, 0) and add exactly 0.
        k0 = 0;
#pragma unroll 1
        for (; k0 < t.nv_exact; k0 += kG) {
            u32x4 xr[kG], gr[kG];
#pragma unroll
            for (int k = 0; k < kG; ++k) gr[k] = load128<true>(pg + (j + ((k0 + k) << lg)));
#pragma unroll
            for (int k = 0; k < kG; ++k) xr[k] = stage[(k0 + k) * kWG + tid];
#pragma unroll
            for (int k = 0; k < kG; ++k) {
                quad(xr[k].x, xr[k].y, gr[k].x, gr[k].y, iv, sc, mul);
                quad(xr[k].z, xr[k].w, gr[k].z, gr[k].w, iv, sc, mul);
            }
        }
#pragma unroll 1
        for (; k0 < t.nv; k0 += kG) {
            u32x4 xr[kG], gr[kG];
#pragma unroll
            for (int k = 0; k < kG; ++k) gr[k] = load128<true>(pg + clamped(k0 + k));
#pragma unroll
            for (int k = 0; k < kG; ++k) xr[k] = stage[(k0 + k) * kWG + tid];
#pragma unroll
            for (int k = 0; k < kG; ++k) {
                const int c = count(k0 + k);
                if (__builtin_amdgcn_ballot_w64(c != kVec) != 0) gr[k] = keep_leading(gr[k], c);
                quad(xr[k].x, xr[k].y, gr[k].x, gr[k].y, iv, sc, mul);
                quad(xr[k].z, xr[k].w, gr[k].z, gr[k].w, iv, sc, mul);
            }
        }
    }
};

#ifndef AMPSENS_FUSED_WAVES
#define AMPSENS_FUSED_WAVES 6
#endif
#ifndef AMPSENS_FUSED_REGS_WAVES
#define AMPSENS_FUSED_REGS_WAVES 6
#endif
// REGS: the variant for units whose threads hold at most kFusedRegNv vectors of a row (tile_regs, no
// dynamic LDS); otherwise rows are staged in LDS (tile).
template <int NF, int F0, int F1, bool POW2, bool REGS>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(REGS ? AMPSENS_FUSED_REGS_WAVES : AMPSENS_FUSED_WAVES,
                                                                    REGS ? AMPSENS_FUSED_REGS_WAVES : AMPSENS_FUSED_WAVES)))
void sens_fused_rows_kernel(const ResolvedUnit* __restrict__ runits, const ChunkRef* __restrict__ map,
                            uint32_t n_chunks, float* __restrict__ partials, int code0, int code1) {
    saturating_fp8_conversions();
    extern __shared__ __attribute__((aligned(16))) unsigned char fused_lds[];   // [nv][kWG] vectors, then 2 * kWaves words
    __shared__ uint32_t red[2 * kWaves];
    __shared__ float scale_table[kScaleTableWords];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    fill_scale_table(scale_table, code0, code1);
    __syncthreads();
    for (uint32_t c = blockIdx.x; c < n_chunks; c += gridDim.x) {
        const ChunkRef ref = map[c];
        const ResolvedUnit u = runits[ref.unit];
        const FusedGeom geo = FusedGeom::unpack(u.head);
        FusedRows<NF, F0, F1, POW2> ctx;
        ctx.x = (gptr16_t)u.x;
        ctx.g = (gptr16_t)u.dx;
        ctx.ts = const_cast<float*>(u.row_scale);
        ctx.ti = const_cast<float*>(u.row_inv);
        ctx.cols = u.cols;
        ctx.code0 = code0;
        ctx.code1 = code1;
        ctx.red = red;
        ctx.scale_table = scale_table;
        ctx.stage = reinterpret_cast<u32x4*>(fused_lds);
        ctx.parity = 0;
#pragma unroll
        for (int f = 0; f < NF; ++f) { ctx.E[f] = 0.0f; ctx.pk[f] = 0; }
        ctx.A = 0.0f;
        FusedTileWalk walk;
        walk.begin(u, geo, ref.local, tid);
        if constexpr (REGS) {
            if (geo.wide) {                              // short dense rows: tiles of 1024 consecutive vectors
                const int64_t total = (int64_t)u.rows << geo.lanes_log2;
                int64_t v0 = (int64_t)ref.local * geo.tiles * (kFusedRegNv * kWG);
                for (int q = 0; q < geo.tiles && v0 < total; ++q, v0 += kFusedRegNv * kWG)
                    ctx.wide_tile(v0, total, geo.lanes_log2);
            } else {
                typename FusedRows<NF, F0, F1, POW2>::Regs r;
                for (FusedTile t = walk.next(); t.valid; t = walk.next()) {
                    ctx.regs_issue(t, r);
                    ctx.regs_finish(t, r);
                }
            }
        } else {
            for (FusedTile t = walk.next(); t.valid; t = walk.next()) ctx.tile(t);
        }
        float v[NF + 1];
#pragma unroll
        for (int f = 0; f < NF; ++f) v[f] = wave_sum(ctx.E[f]);
        v[NF] = wave_sum(ctx.A);
        if (lane == 0) {
            float* slot = partials + ((size_t)ref.slot * kWaves + wave) * (NF + 1);
#pragma unroll
            for (int k = 0; k <= NF; ++k) slot[k] = v[k];
        }
        __syncthreads();                                            // the LDS words are free for the next chunk
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

// ---- launch helpers -----------------------------------------------------------------------------

typedef void (*sens_fn_t)(const ResolvedUnit*, const ChunkRef*, uint32_t, float*);
typedef void (*sens_fused_fn_t)(const ResolvedUnit*, const ChunkRef*, uint32_t, float*, int, int);

template <bool POW2, bool REGS>
sens_fused_fn_t sens_fused_variant_of(int n_fmts, int fmt0, int fmt1) {
    if (n_fmts == 1) return fmt0 == 0 ? sens_fused_rows_kernel<1, 0, 0, POW2, REGS> : sens_fused_rows_kernel<1, 1, 1, POW2, REGS>;
    if (fmt0 == 0) return fmt1 == 0 ? sens_fused_rows_kernel<2, 0, 0, POW2, REGS> : sens_fused_rows_kernel<2, 0, 1, POW2, REGS>;
    return fmt1 == 0 ? sens_fused_rows_kernel<2, 1, 0, POW2, REGS> : sens_fused_rows_kernel<2, 1, 1, POW2, REGS>;
}
// pow2: every format of the call carries the power-of-two scale rule; regs: the class whose rows stay in registers
sens_fused_fn_t sens_fused_variant(int n_fmts, int fmt0, int fmt1, bool pow2, bool regs) {
    if (regs)
        return pow2 ? sens_fused_variant_of<true, true>(n_fmts, fmt0, fmt1) : sens_fused_variant_of<false, true>(n_fmts, fmt0, fmt1);
    return pow2 ? sens_fused_variant_of<true, false>(n_fmts, fmt0, fmt1) : sens_fused_variant_of<false, false>(n_fmts, fmt0, fmt1);
}

template <bool POW2>
sens_fn_t sens_tensor_variant_of(int n_fmts, int fmt0, int fmt1) {
    if (n_fmts == 1) return fmt0 == 0 ? sens_kernel<1, 0, 0, POW2> : sens_kernel<1, 1, 1, POW2>;
    if (fmt0 == 0) return fmt1 == 0 ? sens_kernel<2, 0, 0, POW2> : sens_kernel<2, 0, 1, POW2>;
    return fmt1 == 0 ? sens_kernel<2, 1, 0, POW2> : sens_kernel<2, 1, 1, POW2>;
}

sens_fn_t sens_variant(int n_fmts, int fmt0, int fmt1, int cls, bool pow2 = false) {
    if (cls == 1) {
        if (n_fmts == 1) return fmt0 == 0 ? sens_wrows_kernel<1, 0, 0, false> : sens_wrows_kernel<1, 1, 1, false>;
        if (fmt0 == 0) return fmt1 == 0 ? sens_wrows_kernel<2, 0, 0, false> : sens_wrows_kernel<2, 0, 1, false>;
        return fmt1 == 0 ? sens_wrows_kernel<2, 1, 0, false> : sens_wrows_kernel<2, 1, 1, false>;
    }
    if (cls == 3) {
        if (n_fmts == 1) return fmt0 == 0 ? sens_wrows_kernel<1, 0, 0, true> : sens_wrows_kernel<1, 1, 1, true>;
        if (fmt0 == 0) return fmt1 == 0 ? sens_wrows_kernel<2, 0, 0, true> : sens_wrows_kernel<2, 0, 1, true>;
        return fmt1 == 0 ? sens_wrows_kernel<2, 1, 0, true> : sens_wrows_kernel<2, 1, 1, true>;
    }
    if (cls == 2) {
        if (n_fmts == 1) return fmt0 == 0 ? sens_rows_kernel<1, 0, 0> : sens_rows_kernel<1, 1, 1>;
        if (fmt0 == 0) return fmt1 == 0 ? sens_rows_kernel<2, 0, 0> : sens_rows_kernel<2, 0, 1>;
        return fmt1 == 0 ? sens_rows_kernel<2, 1, 0> : sens_rows_kernel<2, 1, 1>;
    }
    return pow2 ? sens_tensor_variant_of<true>(n_fmts, fmt0, fmt1) : sens_tensor_variant_of<false>(n_fmts, fmt0, fmt1);
}

int resident_blocks(const void* fn, int cus, size_t lds_bytes = 0) {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, kWG, lds_bytes) != hipSuccess || per_cu < 1)
        per_cu = lds_bytes ? 2 : 4;
    return per_cu * cus;
}

}  // namespace

int sens_resident_blocks(int n_fmts, int fmt0, int fmt1, int cls, int cus) {
    if (cls >= kFirstFusedClass)
        return resident_blocks((const void*)sens_fused_variant(n_fmts, fmt0, fmt1, false, cls == kFirstFusedClass), cus,
                               sens_class_lds_bytes(cls));
    const int fit = resident_blocks((const void*)sens_variant(n_fmts, fmt0, fmt1, cls), cus);
    // The kernel for one scale per tensor is compiled for 7 waves per SIMD (the code the compiler writes for
    // 72 registers is the fastest) but runs best on three workgroups per compute unit: 1.640 against 1.665 ms
    // on the config-2 block, 4.35 against 4.42 on config 3, 4.02 against 4.11 on config 4 (two per unit:
    // better on config 3, worse on config 2 and 4; one: far worse).
    if (cls == 0 && fit > 3 * cus) return 3 * cus;
    return fit;
}

typedef void (*sens_w_fn_t)(const WGroup*, uint32_t, uint32_t, const ResolvedUnit*, const uint32_t*, float*);

template <bool ROWS>
static sens_w_fn_t sens_w_variant_of(int n_fmts, int fmt0, int fmt1) {
    if (n_fmts == 1) return fmt0 == 0 ? sens_w_kernel<1, 0, 0, ROWS> : sens_w_kernel<1, 1, 1, ROWS>;
    if (fmt0 == 0) return fmt1 == 0 ? sens_w_kernel<2, 0, 0, ROWS> : sens_w_kernel<2, 0, 1, ROWS>;
    return fmt1 == 0 ? sens_w_kernel<2, 1, 0, ROWS> : sens_w_kernel<2, 1, 1, ROWS>;
}
static sens_w_fn_t sens_w_variant(int n_fmts, int fmt0, int fmt1, int rows) {
    return rows ? sens_w_variant_of<true>(n_fmts, fmt0, fmt1) : sens_w_variant_of<false>(n_fmts, fmt0, fmt1);
}

int sens_w_resident_blocks(int n_fmts, int fmt0, int fmt1, int rows, int cus) {
    const int fit = resident_blocks((const void*)sens_w_variant(n_fmts, fmt0, fmt1, rows), cus);
    // With two formats two workgroups per compute unit stream faster than the four that fit (1.065 against
    // 1.095 ms on the config-2 block, 3.86 against 3.94 on config 4, 0.573 against 0.592 on config 1); with one
    // format they do not (2.70 against 2.26 ms on config 3).
    if (n_fmts == 2 && fit > 2 * cus) return 2 * cus;
    return fit;
}

hipError_t launch_sens_w(const WGroup* d_groups, uint32_t n_groups, uint32_t n_items,
                         const ResolvedUnit* d_runits, const uint32_t* d_chunk_begin, int n_fmts, int fmt0,
                         int fmt1, int rows, float* d_partials, int grid, hipStream_t stream) {
    hipLaunchKernelGGL(sens_w_variant(n_fmts, fmt0, fmt1, rows), dim3(grid), dim3(kWG), 0, stream, d_groups,
                       n_groups, n_items, d_runits, d_chunk_begin, d_partials);
    return hipGetLastError();
}

// Three workgroups per compute unit, not the eight that fit: on a 5.7 GB pass grids of 768 and 1024 workgroups
// read 6 680-6 700 and 6 640-6 660 GB/s, 2048 workgroups 6 480 (grids that are not a multiple of the 256
// compute units fall in between).
int absmax_resident_blocks(int cus) {
    const int fit = resident_blocks((const void*)absmax_kernel, cus);
    return fit < 3 * cus ? fit : 3 * cus;
}
int absmax_rows_resident_blocks(int cus) { return resident_blocks((const void*)absmax_rows_kernel, cus); }

hipError_t launch_absmax_rows(const RowTensor* d_tensors, uint32_t n_tensors, uint32_t n_items,
                              int n_fmts, int fmt0, int fmt1, float* d_amax, float* d_scale,
                              float* d_inv, uint32_t* d_flags, int grid, hipStream_t stream) {
    hipLaunchKernelGGL(zero_u32_kernel, dim3((n_tensors + kWG - 1) / kWG), dim3(kWG), 0, stream, d_flags,
                       n_tensors);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n_items == 0) return e;
    hipLaunchKernelGGL(absmax_rows_kernel, dim3(grid), dim3(kWG), 0, stream, d_tensors, n_tensors, n_items,
                       n_fmts, fmt0, fmt1, d_amax, d_scale, d_inv, d_flags);
    return hipGetLastError();
}

hipError_t launch_table_write(const void* host_src, size_t bytes, void* d_dst, hipStream_t stream) {
    const uint8_t* src = (const uint8_t*)host_src;
    uint8_t* dst = (uint8_t*)d_dst;
    TablePiece piece;
    for (size_t off = 0; off < bytes; off += sizeof(TablePiece)) {
        const size_t n = bytes - off < sizeof(TablePiece) ? bytes - off : sizeof(TablePiece);
        std::memcpy(&piece, src + off, n);
        if (n % 16) std::memset((uint8_t*)&piece + n, 0, 16 - n % 16);
        hipLaunchKernelGGL(table_write_kernel, dim3(1), dim3(kWG), 0, stream, piece, (uint4*)(dst + off),
                           (uint32_t)((n + 15) / 16));
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_table_runs(const TableRun* host_runs, size_t n, void* d_table, size_t off_schedule,
                             hipStream_t stream) {
    TablePiece piece;
    for (size_t i = 0; i < n; i += kRunsPerPiece) {
        const size_t m = n - i < (size_t)kRunsPerPiece ? n - i : (size_t)kRunsPerPiece;
        std::memcpy(&piece, host_runs + i, m * sizeof(TableRun));
        hipLaunchKernelGGL(table_runs_kernel, dim3((unsigned)m), dim3(64), 0, stream, piece, (uint8_t*)d_table,
                           (uint32_t)off_schedule);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_table_literals(const TableLiteral* host_literals, size_t n, void* d_table, size_t off_schedule,
                                 hipStream_t stream) {
    TablePiece piece;
    for (size_t i = 0; i < n; i += kLiteralsPerPiece) {
        const size_t m = n - i < (size_t)kLiteralsPerPiece ? n - i : (size_t)kLiteralsPerPiece;
        std::memcpy(&piece, host_literals + i, m * sizeof(TableLiteral));
        hipLaunchKernelGGL(table_literals_kernel, dim3((unsigned)m), dim3(64), 0, stream, piece, (uint8_t*)d_table,
                           (uint32_t)off_schedule);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_small_setup(const void* host_src, size_t bytes, void* d_dst, size_t off_cb, size_t off_schedule,
                              uint32_t n_units, uint32_t n_chunks, ResolvedUnit* d_runits, ChunkRef* d_map,
                              int resolve_fmts, hipStream_t stream) {
    if (bytes > sizeof(TablePiece) || n_chunks > kSmallSetupChunks) return hipErrorInvalidValue;
    TablePiece piece;
    std::memcpy(&piece, host_src, bytes);
    if (bytes % 16) std::memset((uint8_t*)&piece + bytes, 0, 16 - bytes % 16);
    hipLaunchKernelGGL(small_setup_kernel, dim3(1), dim3(kWG), 0, stream, piece, (uint32_t)((bytes + 15) / 16),
                       (uint4*)d_dst, (uint32_t)off_cb, (uint32_t)off_schedule, n_units, n_chunks, d_runits, d_map,
                       resolve_fmts);
    return hipGetLastError();
}

hipError_t launch_prepare(const WorkUnit* d_units, const uint32_t* d_chunk_begin,
                          const UnitSchedule* d_schedule, uint32_t n_units, uint32_t n_chunks,
                          ResolvedUnit* d_runits, ChunkRef* d_map, hipStream_t stream) {
    const uint32_t n = n_units > n_chunks ? n_units : n_chunks;
    hipLaunchKernelGGL(prepare_kernel, dim3((n + kWG - 1) / kWG), dim3(kWG), 0, stream, d_units,
                       d_chunk_begin, d_schedule, n_units, n_chunks, d_runits, d_map);
    return hipGetLastError();
}

hipError_t launch_resolve(const WorkUnit* d_units, uint32_t n_units, int n_fmts, ResolvedUnit* d_runits,
                          hipStream_t stream) {
    hipLaunchKernelGGL(resolve_kernel, dim3((n_units + kWG - 1) / kWG), dim3(kWG), 0, stream, d_units, n_units,
                       n_fmts, d_runits);
    return hipGetLastError();
}

hipError_t launch_absmax(const ResolvedUnit* d_runits, const ChunkRef* d_map, uint32_t n_chunks,
                         uint32_t* d_partial_max, int grid, hipStream_t stream) {
    hipLaunchKernelGGL(absmax_kernel, dim3(grid), dim3(kWG), 0, stream, d_runits, d_map, n_chunks,
                       d_partial_max);
    return hipGetLastError();
}

hipError_t launch_absmax_finalize(const uint32_t* d_chunk_begin, const uint32_t* d_partial_max,
                                  int n_tensors, int n_fmts, int fmt0, int fmt1, float* d_amax,
                                  float* d_scale, float* d_inv, uint32_t* d_flags,
                                  hipStream_t stream) {
    hipLaunchKernelGGL(absmax_finalize_kernel, dim3(n_tensors), dim3(kFinThreads), 0, stream, d_chunk_begin,
                       d_partial_max, n_fmts, fmt0, fmt1, d_amax, d_scale, d_inv, d_flags);
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

hipError_t launch_sens(const ResolvedUnit* d_runits, const ChunkRef* d_map, uint32_t n_chunks,
                       int n_fmts, int fmt0, int fmt1, int cls, float* d_partials, int grid,
                       hipStream_t stream) {
    // the scaled conversions serve calls whose formats all carry the power-of-two scale rule
    const bool pow2 = (fmt0 & kScalePow2) != 0 && (fmt1 & kScalePow2) != 0;
    if (cls >= kFirstFusedClass)
        hipLaunchKernelGGL(sens_fused_variant(n_fmts, fmt0 & 0xFF, fmt1 & 0xFF, pow2, cls == kFirstFusedClass), dim3(grid), dim3(kWG),
                           sens_class_lds_bytes(cls), stream, d_runits, d_map, n_chunks, d_partials, fmt0, fmt1);
    else
        hipLaunchKernelGGL(sens_variant(n_fmts, fmt0 & 0xFF, fmt1 & 0xFF, cls, pow2), dim3(grid), dim3(kWG), 0, stream,
                           d_runits, d_map, n_chunks, d_partials);
    return hipGetLastError();
}

hipError_t launch_sens_finalize(const ResolvedUnit* d_runits, const uint32_t* d_chunk_begin,
                                uint32_t n_units, int n_fmts, const float* d_partials,
                                float* d_out, hipStream_t stream) {
    const dim3 grid(n_units);
    if (n_fmts == 1)
        hipLaunchKernelGGL(sens_finalize_kernel<1>, grid, dim3(kWG), 0, stream, d_runits,
                           d_chunk_begin, n_units, d_partials, d_out);
    else
        hipLaunchKernelGGL(sens_finalize_kernel<2>, grid, dim3(kWG), 0, stream, d_runits,
                           d_chunk_begin, n_units, d_partials, d_out);
    return hipGetLastError();
}

}  // namespace ampsens
