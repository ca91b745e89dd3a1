// Device-side building blocks shared by the gfx950 kernel files: packed loads and stores of a
// lane's 8 consecutive entries, bfloat16 conversion, DPP wave reductions, tile geometry and the
// complete update of a 1-D parameter by one workgroup.  Everything has internal linkage.
#pragma once

#include <hip/hip_runtime.h>

#include "came_kernels.h"

namespace came {
namespace {

using f32x4 = float __attribute__((ext_vector_type(4)));
using u32x4 = uint32_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bits_to_float(uint32_t b) { return __uint_as_float(b); }

// The caller's parameter and gradient addresses reach the kernels through a pointer table in
// device memory, so the compiler cannot know they are global-memory addresses and would use
// FLAT loads and stores for them.  Those count against the LDS counter as well and may
// complete out of order, so every wait on one of them (and every wait for an LDS read while
// one is in flight) becomes a wait for ALL outstanding memory operations -- which undoes the
// software prefetch of the sweeps.  Every access to a caller's buffer therefore goes through a
// pointer in the global address space (what the host guarantees anyway: device memory).
#define CAME_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ CAME_GLOBAL T* glob(T* p)
{
    return (CAME_GLOBAL T*)p;
}

// ---------------------------------------------------------------- loads / stores

template <bool BF16>
__device__ __forceinline__ float load_grad1(const void* g, int64_t idx)
{
    if constexpr (BF16)
        return bits_to_float(static_cast<uint32_t>(glob(static_cast<const uint16_t*>(g))[idx]) << 16);
    else
        return glob(static_cast<const float*>(g))[idx];
}

// A lane's 8 consecutive entries of one row, as they sit in memory.  Kept packed
// between the load and its use so that the next rows' loads can be issued before
// the current rows are consumed (the wait lands at the unpack, not at the load).
template <bool BF16> struct GradRaw;
template <> struct GradRaw<true>  { u32x4 v; };      // 8 bfloat16
template <> struct GradRaw<false> { f32x4 a, b; };   // 8 binary32
struct F32Raw { f32x4 a, b; };

// ALIGNED: every row starts 16-byte aligned (m % 8 == 0) and ncol is 0 or 8: vector
// accesses.  Otherwise the address is only element-aligned: lanes whose 8 columns all exist
// copy them in one go (the compiler chooses the access width the alignment allows), the lane
// at the matrix's right edge goes element by element with bounds.
// NT: non-temporal (streaming) loads, for data read once per sweep and never written.
template <bool BF16, bool ALIGNED, bool NT = true>
__device__ __forceinline__ GradRaw<BF16> load_grad_raw(const void* g, int64_t idx, int ncol)
{
    GradRaw<BF16> r;
    if constexpr (BF16) {
        r.v = u32x4{0u, 0u, 0u, 0u};
        const CAME_GLOBAL uint16_t* p = glob(static_cast<const uint16_t*>(g)) + idx;
        if constexpr (ALIGNED) {
            // gradients are read once per sweep and never written: stream them (measured: sweep 2
            // 6 % faster; the same hint on the M / theta loads or on the stores is slower)
            if (ncol > 0) {
                if constexpr (NT) r.v = __builtin_nontemporal_load((const CAME_GLOBAL u32x4*)p);
                else r.v = *(const CAME_GLOBAL u32x4*)p;
            }
        } else if (ncol == kLaneCols) {
            // all 8 entries exist but the address is only element-aligned: a plain copy lets the
            // compiler pick the widest access the target allows for that alignment
            __builtin_memcpy(&r.v, (const void*)p, sizeof(r.v));
        } else {
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (e < ncol) w[e >> 1] |= static_cast<uint32_t>(p[e]) << ((e & 1) * 16);
            r.v = u32x4{w[0], w[1], w[2], w[3]};
        }
    } else {
        r.a = f32x4{0.f, 0.f, 0.f, 0.f};
        r.b = r.a;
        const CAME_GLOBAL float* p = glob(static_cast<const float*>(g)) + idx;
        if constexpr (ALIGNED) {
            if (ncol > 0) {
                if constexpr (NT) {
                    r.a = __builtin_nontemporal_load((const CAME_GLOBAL f32x4*)p);
                    r.b = __builtin_nontemporal_load((const CAME_GLOBAL f32x4*)p + 1);
                } else {
                    r.a = ((const CAME_GLOBAL f32x4*)p)[0];
                    r.b = ((const CAME_GLOBAL f32x4*)p)[1];
                }
            }
        } else if (ncol == kLaneCols) {
            __builtin_memcpy(&r.a, (const void*)p, sizeof(r.a));
            __builtin_memcpy(&r.b, (const void*)(p + 4), sizeof(r.b));
        } else {
            float w[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) w[e] = e < ncol ? p[e] : 0.f;
            r.a = f32x4{w[0], w[1], w[2], w[3]};
            r.b = f32x4{w[4], w[5], w[6], w[7]};
        }
    }
    return r;
}

// Split ownership: the lane's 8 entries are 4 consecutive ones at element ia and 4 at element ib
// (16-byte aligned as binary32, 8-byte aligned as bfloat16).  Used by the kernels for 16-byte
// aligned rows, where lane l of a tile holds columns 4l..4l+3 and 256+4l..256+4l+3: every
// 16-byte-per-lane instruction on a binary32 array then touches 1 KB contiguous instead of every
// other 16 bytes of 2 KB, which matters for streaming loads (a line that two streaming
// instructions each use half of is requested twice; sweep 1 on binary32 gradients is 10 % faster
// this way, and with bfloat16 gradients the sweeps still gain 0.5-3 %).
// The pair unpacks to x[0..3] (first group) and x[4..7] (second group) like any other GradRaw.
using u32x2 = uint32_t __attribute__((ext_vector_type(2)));

template <bool BF16, bool NT>
__device__ __forceinline__ GradRaw<BF16> load_pair(const void* base, int64_t ia, int64_t ib)
{
    GradRaw<BF16> r;
    if constexpr (BF16) {
        const CAME_GLOBAL uint16_t* p = glob(static_cast<const uint16_t*>(base));
        u32x2 a, b;
        if constexpr (NT) {
            a = __builtin_nontemporal_load((const CAME_GLOBAL u32x2*)(p + ia));
            b = __builtin_nontemporal_load((const CAME_GLOBAL u32x2*)(p + ib));
        } else {
            a = *(const CAME_GLOBAL u32x2*)(p + ia);
            b = *(const CAME_GLOBAL u32x2*)(p + ib);
        }
        r.v = u32x4{a.x, a.y, b.x, b.y};
    } else {
        const CAME_GLOBAL float* p = glob(static_cast<const float*>(base));
        if constexpr (NT) {
            r.a = __builtin_nontemporal_load((const CAME_GLOBAL f32x4*)(p + ia));
            r.b = __builtin_nontemporal_load((const CAME_GLOBAL f32x4*)(p + ib));
        } else {
            r.a = *(const CAME_GLOBAL f32x4*)(p + ia);
            r.b = *(const CAME_GLOBAL f32x4*)(p + ib);
        }
    }
    return r;
}

template <bool BF16>
__device__ __forceinline__ void unpack(const GradRaw<BF16>& r, float (&x)[8])
{
    if constexpr (BF16) {
        x[0] = bits_to_float(r.v.x << 16); x[1] = bits_to_float(r.v.x & 0xffff0000u);
        x[2] = bits_to_float(r.v.y << 16); x[3] = bits_to_float(r.v.y & 0xffff0000u);
        x[4] = bits_to_float(r.v.z << 16); x[5] = bits_to_float(r.v.z & 0xffff0000u);
        x[6] = bits_to_float(r.v.w << 16); x[7] = bits_to_float(r.v.w & 0xffff0000u);
    } else {
        x[0] = r.a.x; x[1] = r.a.y; x[2] = r.a.z; x[3] = r.a.w;
        x[4] = r.b.x; x[5] = r.b.y; x[6] = r.b.z; x[7] = r.b.w;
    }
}

__device__ __forceinline__ void unpack(const F32Raw& r, float (&x)[8])
{
    x[0] = r.a.x; x[1] = r.a.y; x[2] = r.a.z; x[3] = r.a.w;
    x[4] = r.b.x; x[5] = r.b.y; x[6] = r.b.z; x[7] = r.b.w;
}

template <bool ALIGNED>
__device__ __forceinline__ F32Raw load_f32_raw(const float* base, int64_t idx, int ncol)
{
    F32Raw r;
    r.a = f32x4{0.f, 0.f, 0.f, 0.f};
    r.b = r.a;
    const CAME_GLOBAL float* p = glob(base) + idx;
    if constexpr (ALIGNED) {
        if (ncol > 0) {
            r.a = ((const CAME_GLOBAL f32x4*)p)[0];
            r.b = ((const CAME_GLOBAL f32x4*)p)[1];
        }
    } else if (ncol == kLaneCols) {
        __builtin_memcpy(&r.a, (const void*)p, sizeof(r.a));
        __builtin_memcpy(&r.b, (const void*)(p + 4), sizeof(r.b));
    } else {
        float w[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = e < ncol ? p[e] : 0.f;
        r.a = f32x4{w[0], w[1], w[2], w[3]};
        r.b = f32x4{w[4], w[5], w[6], w[7]};
    }
    return r;
}

template <bool ALIGNED>
__device__ __forceinline__ void store_f32x8(float* base, int64_t idx, int ncol, const float (&x)[8])
{
    CAME_GLOBAL float* p = glob(base) + idx;
    if constexpr (ALIGNED) {
        if (ncol > 0) {
            ((CAME_GLOBAL f32x4*)p)[0] = f32x4{x[0], x[1], x[2], x[3]};
            ((CAME_GLOBAL f32x4*)p)[1] = f32x4{x[4], x[5], x[6], x[7]};
        }
    } else if (ncol == kLaneCols) {
        const f32x4 a = {x[0], x[1], x[2], x[3]}, b = {x[4], x[5], x[6], x[7]};
        __builtin_memcpy((void*)p, &a, sizeof(a));
        __builtin_memcpy((void*)(p + 4), &b, sizeof(b));
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < ncol) p[e] = x[e];
    }
}

// binary32 -> bfloat16, round to nearest even; NaN stays NaN (quiet bit forced).
__device__ __forceinline__ uint32_t bf16_bits(float x)
{
    const uint32_t u = __float_as_uint(x);
    const uint32_t rounded = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    return (u & 0x7fffffffu) > 0x7f800000u ? ((u >> 16) | 0x40u) : rounded;
}

// Stores 8 values as bfloat16 at element idx of a bfloat16 array (same alignment rules
// as the binary32 stores: vector store when ALIGNED, element-wise with bounds otherwise).
template <bool ALIGNED>
__device__ __forceinline__ void store_bf16x8(void* base, int64_t idx, int ncol, const float (&x)[8])
{
    CAME_GLOBAL uint16_t* p = glob(static_cast<uint16_t*>(base)) + idx;
    if constexpr (ALIGNED) {
        if (ncol > 0) {
            u32x4 v;
            v.x = bf16_bits(x[0]) | (bf16_bits(x[1]) << 16);
            v.y = bf16_bits(x[2]) | (bf16_bits(x[3]) << 16);
            v.z = bf16_bits(x[4]) | (bf16_bits(x[5]) << 16);
            v.w = bf16_bits(x[6]) | (bf16_bits(x[7]) << 16);
            *(CAME_GLOBAL u32x4*)p = v;
        }
    } else if (ncol == kLaneCols) {
        u32x4 v;
        v.x = bf16_bits(x[0]) | (bf16_bits(x[1]) << 16);
        v.y = bf16_bits(x[2]) | (bf16_bits(x[3]) << 16);
        v.z = bf16_bits(x[4]) | (bf16_bits(x[5]) << 16);
        v.w = bf16_bits(x[6]) | (bf16_bits(x[7]) << 16);
        __builtin_memcpy((void*)p, &v, sizeof(v));
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < ncol) p[e] = static_cast<uint16_t>(bf16_bits(x[e]));
    }
}

__device__ __forceinline__ F32Raw load_f32_pair(const float* base, int64_t ia, int64_t ib)
{
    F32Raw r;
    const CAME_GLOBAL float* p = glob(base);
    r.a = *(const CAME_GLOBAL f32x4*)(p + ia);
    r.b = *(const CAME_GLOBAL f32x4*)(p + ib);
    return r;
}

// oka / okb: whether the first / second group is stored at all.
__device__ __forceinline__ void store_f32_pair(float* base, int64_t ia, int64_t ib, bool oka, bool okb, const float (&x)[8])
{
    CAME_GLOBAL float* p = glob(base);
    if (oka) *(CAME_GLOBAL f32x4*)(p + ia) = f32x4{x[0], x[1], x[2], x[3]};
    if (okb) *(CAME_GLOBAL f32x4*)(p + ib) = f32x4{x[4], x[5], x[6], x[7]};
}

__device__ __forceinline__ void store_bf16_pair(void* base, int64_t ia, int64_t ib, bool oka, bool okb, const float (&x)[8])
{
    CAME_GLOBAL uint16_t* p = glob(static_cast<uint16_t*>(base));
    u32x2 a, b;
    a.x = bf16_bits(x[0]) | (bf16_bits(x[1]) << 16); a.y = bf16_bits(x[2]) | (bf16_bits(x[3]) << 16);
    b.x = bf16_bits(x[4]) | (bf16_bits(x[5]) << 16); b.y = bf16_bits(x[6]) | (bf16_bits(x[7]) << 16);
    if (oka) *(CAME_GLOBAL u32x2*)(p + ia) = a;
    if (okb) *(CAME_GLOBAL u32x2*)(p + ib) = b;
}

// The momentum as stored: binary32, or bfloat16 (MB16) widened exactly on load and rounded
// to nearest even on store.  `M` is the tensor's momentum array inside the state blob; idx
// counts elements.  Plain cached accesses: sweep 3 re-reads what sweep 2 read.
template <bool MB16, bool ALIGNED>
__device__ __forceinline__ GradRaw<MB16> load_mom_raw(const float* M, int64_t idx, int ncol)
{
    return load_grad_raw<MB16, ALIGNED, false>(M, idx, ncol);
}

template <bool MB16, bool ALIGNED>
__device__ __forceinline__ void store_mom(float* M, int64_t idx, int ncol, const float (&x)[8])
{
    if constexpr (MB16) store_bf16x8<ALIGNED>(M, idx, ncol, x);
    else store_f32x8<ALIGNED>(M, idx, ncol, x);
}

__device__ __forceinline__ float load_mom1(const float* M, int64_t i, bool mb16)
{
    return mb16 ? bits_to_float(static_cast<uint32_t>(glob(reinterpret_cast<const uint16_t*>(M))[i]) << 16) : glob(M)[i];
}

__device__ __forceinline__ void store_mom1(float* M, int64_t i, bool mb16, float x)
{
    if (mb16) glob(reinterpret_cast<uint16_t*>(M))[i] = static_cast<uint16_t>(bf16_bits(x));
    else glob(M)[i] = x;
}

// ---------------------------------------------------------------- reductions

// DPP controls (GFX9 encoding): quad_perm [1,0,3,2], quad_perm [2,3,0,1], mirror within
// 8 lanes, mirror within 16 lanes, lane 15 of a row to the next row, lane 31 to rows 2-3.
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140,
              kDppBcast15 = 0x142, kDppBcast31 = 0x143;

// Value of `v` in the lane that DPP control CTRL designates as this lane's source; lanes
// without a source (rows that a row broadcast does not reach) read 0 (bound_ctrl).  The
// "old" operand is left undefined on purpose: every lane either has a source or takes
// the bound_ctrl zero, and an explicit old = 0 would cost a register move per use.
template <int CTRL>
__device__ __forceinline__ float dpp_get(float v)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}

template <int CTRL>
__device__ __forceinline__ double dpp_get(double v)
{
    const int lo = __builtin_amdgcn_mov_dpp(__double2loint(v), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(v), CTRL, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes of a wave; the total is valid in LANE 63 ONLY.  Four butterfly
// steps inside each row of 16 lanes, then two row broadcasts; all DPP, no LDS traffic.
// After the butterflies every lane of row k holds t_k.  Broadcast 15 (lane 15 of each
// row to the whole next row; row 0 receives 0) leaves t0, t0+t1, t1+t2, t2+t3; broadcast
// 31 (lane 31 to rows 2 and 3; rows 0, 1 receive 0) then makes row 3 = t0+t1+t2+t3.
// Fixed order, hence deterministic.  Every lane of the wave must be active.
template <class T>
__device__ __forceinline__ T wave_sum_lane63(T v)
{
    v += dpp_get<kDppXor1>(v);
    v += dpp_get<kDppXor2>(v);
    v += dpp_get<kDppHalfMirror>(v);
    v += dpp_get<kDppMirror>(v);
    v += dpp_get<kDppBcast15>(v);
    v += dpp_get<kDppBcast31>(v);
    return v;
}

__device__ __forceinline__ double lane63_to_all(double v)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double wave_sum(double v) { return lane63_to_all(wave_sum_lane63(v)); }

// Sum over the 256 threads of a workgroup, same value returned to every thread.
// Fixed tree, hence deterministic.  lds4: 4 doubles of LDS, reusable afterwards.
__device__ __forceinline__ double block_sum(double v, double* lds4)
{
    v = wave_sum_lane63(v);
    if ((threadIdx.x & 63) == 63) lds4[threadIdx.x >> 6] = v;
    __syncthreads();
    const double total = (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
    __syncthreads();
    return total;
}

// Sum of a short list of doubles (a few hundred at most), computed by one wave in a
// fixed order; every wave that evaluates it gets the same bits.
__device__ __forceinline__ double wave_sum_list(const double* list, int count)
{
    double s = 0.0;
    for (int k = threadIdx.x & 63; k < count; k += 64) s += list[k];
    return wave_sum(s);
}

struct TileGeom {
    int lane, wave;
    int64_t row0;
    int nrows;
    int64_t col;  // first column of this lane
    int ncol;     // valid columns of this lane: 0..8
};

// `tile_rows`: the height of the row blocks that it.rb counts (TensorMeta.tile_rows for the items
// of sweeps 1 and 2, TensorMeta.tile_rows3 for the update sweep's).
__device__ __forceinline__ TileGeom tile_geom(const TensorMeta& tm, const WorkItem& it, int32_t tile_rows)
{
    TileGeom t;
    t.lane = threadIdx.x & 63;
    t.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    t.row0 = static_cast<int64_t>(it.rb) * tile_rows;
    const int64_t left = tm.n - t.row0;
    t.nrows = static_cast<int>(left < tile_rows ? left : tile_rows);
    t.col = static_cast<int64_t>(it.cb) * kTileCols + t.lane * kLaneCols;
    const int64_t cleft = tm.m - t.col;
    t.ncol = cleft >= kLaneCols ? kLaneCols : (cleft > 0 ? static_cast<int>(cleft) : 0);
    return t;
}

__device__ __forceinline__ TileGeom tile_geom(const TensorMeta& tm, const WorkItem& it)
{
    return tile_geom(tm, it, tm.tile_rows);
}

// Tile of a folded matrix (work items of kinds 5 and 6): row0 and nrows count rows of the view with
// ceil(n/2) rows of 2m columns.  All 512 columns of the tile exist; which columns of the matrix a
// lane holds is split_geom's business.
__device__ __forceinline__ TileGeom folded_geom(const TensorMeta& tm, const WorkItem& it, int32_t tile_rows)
{
    TileGeom t;
    t.lane = threadIdx.x & 63;
    t.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    t.row0 = static_cast<int64_t>(it.rb) * tile_rows;
    const int64_t left = (tm.n + 1) / 2 - t.row0;
    t.nrows = static_cast<int>(left < tile_rows ? left : tile_rows);
    t.col = static_cast<int64_t>(it.cb) * kTileCols + t.lane * kLaneCols;
    t.ncol = kLaneCols;
    return t;
}

// ---------------------------------------------------------------- vectors

// Algorithm 2 on a 1-D parameter (n x 1 special case: v = r, s = R).  One
// workgroup owns the whole vector; the RMS of Eq. 1 is a workgroup reduction.
template <bool BF16>
__device__ void vector_update(const TensorMeta& tm, const void* __restrict__ g, float* __restrict__ theta,
                              uint16_t* __restrict__ theta16, float* state,
                              const SweepHyper& h, const FinalizeHyper& fh, TensorScalars* sc,
                              double* lds4)
{
    // the arrays of one tensor never overlap (the host checks the caller's buffers): say so, so
    // that the loads of several iterations can be in flight instead of waiting for each store
    float* __restrict__ M = state + tm.off_M;
    float* __restrict__ v = state + tm.off_r;
    float* __restrict__ s = state + tm.off_R;
    const int64_t n = tm.n;
    const bool mb16 = tm.flags & kFlagBf16Momentum;
    const bool came = h.algo == CAME_ALGO_CAME && !(tm.flags & kFlagMomentumOnly);
    double acc = 0.0;
#pragma unroll 4
    for (int64_t i = threadIdx.x; i < n; i += kWorkgroup) {
        const float gi = load_grad1<BF16>(g, i);
        const float vi = h.beta2 * v[i] + h.one_minus_beta2 * (gi * gi + h.eps1);
        v[i] = vi;
        const float u = gi * rsqrtf(vi);
        acc += static_cast<double>(u) * static_cast<double>(u);
    }
    const double P = block_sum(acc, lds4);
    const double rms = sqrt(P / static_cast<double>(n));
    const double denom = fmax(1.0, rms / fh.clip_d);
    const float kappa = static_cast<float>(1.0 / denom);
    if (threadIdx.x == 0) {
        sc->kappa = kappa;
        sc->rms_u = static_cast<float>(rms);
    }
#pragma unroll 4
    for (int64_t i = threadIdx.x; i < n; i += kWorkgroup) {
        const float gi = load_grad1<BF16>(g, i);
        const float uh = kappa * (gi * rsqrtf(v[i]));
        const float Mi = fmaf(h.beta1, load_mom1(M, i, mb16), h.one_minus_beta1 * uh);
        store_mom1(M, i, mb16, Mi);
        float tn;
        if (came) {
            const float dU = uh - Mi;
            const float si = h.beta3 * s[i] + h.one_minus_beta3 * (dU * dU + h.eps2);
            s[i] = si;
            tn = fmaf(glob(theta)[i], h.decay, -(h.lr * Mi * rsqrtf(si)));
        } else {
            tn = fmaf(glob(theta)[i], h.decay, -(h.lr * Mi));
        }
        glob(theta)[i] = tn;
        if (theta16) glob(theta16)[i] = static_cast<uint16_t>(bf16_bits(tn));
    }
}

// Work item `item` is a whole 1-D parameter: its complete update by this workgroup.
__device__ __forceinline__ void vector_item(const DeviceTables& tb, int32_t item, const SweepHyper& h,
                                            const FinalizeHyper& fh, double* lds4)
{
    const WorkItem it = tb.items[item];
    const TensorMeta& tm = tb.metas[it.tensor];
    const void* g = tb.grad[it.tensor];
    float* theta = static_cast<float*>(tb.theta[it.tensor]);
    uint16_t* theta16 = static_cast<uint16_t*>(tb.theta16[it.tensor]);
    if (tm.flags & kFlagBf16Grad) vector_update<true>(tm, g, theta, theta16, tb.state, h, fh, tb.scalars + it.tensor, lds4);
    else                          vector_update<false>(tm, g, theta, theta16, tb.state, h, fh, tb.scalars + it.tensor, lds4);
}

// Split ownership (see load_pair): where a lane's two groups of 4 columns lie.  va, vb: first
// column of each group in the tile's view (the matrix, or the ceil(n/2) x 2m view of a folded
// one); ha, hb: folded tiles, which row of a pair each group lies in -- the same for every lane of
// a tile, since the view's rows change over at a multiple of 256 columns; ca, cb: first column of
// each group in the matrix.
struct SplitGeom {
    int64_t va, vb, ca, cb;
    int ha, hb;
};

template <bool FOLDED>
__device__ __forceinline__ SplitGeom split_geom(const TensorMeta& tm, const WorkItem& it, const TileGeom& t)
{
    SplitGeom g;
    g.va = static_cast<int64_t>(it.cb) * kTileCols + 4 * t.lane;
    g.vb = g.va + kTileCols / 2;
    if constexpr (FOLDED) {
        const int k = static_cast<int>(tm.m / kTileCols);  // the column block that spans both rows of a pair
        g.ha = it.cb > k ? 1 : 0;
        g.hb = it.cb >= k ? 1 : 0;
    } else {
        g.ha = g.hb = 0;
    }
    g.ca = g.va - g.ha * tm.m;
    g.cb = g.vb - g.hb * tm.m;
    return g;
}

// Element indices of the lane's two groups in step j of its wave, and whether their rows exist
// (folded matrices with an odd number of rows: the last pair has no second row; its lanes then
// read the first row again and their data is discarded).
struct SplitStep {
    int64_t ia, ib;
    bool oka, okb;
    int rowa, rowb;  // rows of the matrix, counted from the tile's first
};

template <bool FOLDED>
__device__ __forceinline__ SplitStep split_step(const TileGeom& t, const SplitGeom& g, int j, int64_t pitch, int mrows, int64_t m)
{
    SplitStep s;
    const int64_t base = (t.row0 + t.wave + kWaves * j) * pitch;
    s.ia = base + g.va;
    s.ib = base + g.vb;
    if constexpr (FOLDED) {
        const int first = 2 * (t.wave + kWaves * j);
        s.rowa = first + g.ha;
        s.rowb = first + g.hb;
        s.oka = s.rowa < mrows;
        s.okb = s.rowb < mrows;
        if (!s.oka) s.ia -= m;
        if (!s.okb) s.ib -= m;
    } else {
        s.rowa = s.rowb = t.wave + kWaves * j;
        s.oka = s.okb = true;
    }
    return s;
}

// LDS slot (column of the tile's view) of entry e of a lane under split ownership.
__device__ __forceinline__ int split_slot(int lane, int e)
{
    return e < 4 ? 4 * lane + e : kTileCols / 2 + 4 * lane + (e - 4);
}

// Column this lane loads from: its own, or (overhanging lanes of a ragged tile) the
// tile's first columns, which exist because the tile exists and m % 8 == 0.
template <bool FULL>
__device__ __forceinline__ int64_t load_col(const TileGeom& t, int cb)
{
    if constexpr (FULL) return t.col;
    else return t.ncol > 0 ? t.col : static_cast<int64_t>(cb) * kTileCols;
}

}  // namespace
}  // namespace came
