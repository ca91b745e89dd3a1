// gfx950 kernels of the CAME step (Algorithm 2 of the CAME paper).
//
// One step is five grouped launches over ALL tensors of a group:
//
//   sweep 1    g            -> row/column partial sums of g^2          (r_t, c_t lines)
//   finalize 1 partials     -> r_t, c_t, sqrt(1^T r_t)
//   sweep 2    g, M_{t-1}   -> row/column partial sums of u^2, u M, M^2 with u = g / sqrt(v_t)
//   finalize 2 partials     -> kappa = 1/max(1, RMS(u_t)/d) (Eq. 1), R_t, C_t, sqrt(1^T R_t)
//   sweep 3    g, M, theta  -> M_t, theta_t
//
// v_t = r c^T / (1^T r) and S_t = R C^T / (1^T R) are never materialised:
//   1/sqrt(v_ij) = rsqrt(r_i) * sqrt(1^T r) * rsqrt(c_j)
// and likewise for S, so the per-element work has no division or square root
// and the product r_i c_j (which can leave the binary32 range for all-zero
// rows regularised only by eps1) is never formed.
//
// Sweep 2 gets the statistics of the instability U_t = (u^_t - M_t)^2 BEFORE
// kappa and M_t exist, from M_t = beta1 M_{t-1} + (1-beta1) u^_t:
//   u^ - M_t = beta1 (u^ - M_{t-1})   =>   U = beta1^2 (kappa u - M_{t-1})^2
//   sum U = beta1^2 (kappa^2 sum u^2 - 2 kappa sum u M_{t-1} + sum M_{t-1}^2).
// The three sums cancel when u^ is close to M_{t-1}, so they are accumulated in
// binary64 from exact products of binary32 values; finalize 2 combines them.
//
// Tile: 4 wave64s sweep `tile_rows` rows of a 512-column stripe; lane l owns
// columns 8l..8l+7 (one 16-byte bf16 load, two 16-byte f32 loads), wave w rows
// w, w+4, ...  Row sums: 8 in-lane adds, then a wave reduction.  Column sums:
// per-lane accumulators down the tile, combined across the 4 waves in LDS and
// written per (row block, column); the finalize kernels add the row blocks.
// No atomics on data: results are bit-reproducible run to run.
#include <hip/hip_runtime.h>

#include "came_kernels.h"

namespace came {
namespace {

using f32x4 = float __attribute__((ext_vector_type(4)));
using u32x4 = uint32_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bits_to_float(uint32_t b) { return __uint_as_float(b); }

// ---------------------------------------------------------------- loads / stores

template <bool BF16>
__device__ __forceinline__ float load_grad1(const void* g, int64_t idx)
{
    if constexpr (BF16)
        return bits_to_float(static_cast<uint32_t>(static_cast<const uint16_t*>(g)[idx]) << 16);
    else
        return static_cast<const float*>(g)[idx];
}

// 8 consecutive gradient entries starting at element idx, widened to binary32.
// ALIGNED: the caller guarantees ncol is 0 or 8 and idx % 8 == 0 with a 16-byte aligned base.
template <bool BF16, bool ALIGNED>
__device__ __forceinline__ void load_grad8(const void* g, int64_t idx, int ncol, float (&x)[8])
{
    if constexpr (ALIGNED) {
        if (ncol > 0) {
            if constexpr (BF16) {
                const u32x4 raw = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(g) + idx);
                x[0] = bits_to_float(raw.x << 16); x[1] = bits_to_float(raw.x & 0xffff0000u);
                x[2] = bits_to_float(raw.y << 16); x[3] = bits_to_float(raw.y & 0xffff0000u);
                x[4] = bits_to_float(raw.z << 16); x[5] = bits_to_float(raw.z & 0xffff0000u);
                x[6] = bits_to_float(raw.w << 16); x[7] = bits_to_float(raw.w & 0xffff0000u);
            } else {
                const f32x4* p = reinterpret_cast<const f32x4*>(static_cast<const float*>(g) + idx);
                const f32x4 a = p[0], b = p[1];
                x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
                x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = 0.f;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = e < ncol ? load_grad1<BF16>(g, idx + e) : 0.f;
    }
}

template <bool ALIGNED>
__device__ __forceinline__ void load_f32x8(const float* base, int64_t idx, int ncol, float (&x)[8])
{
    if constexpr (ALIGNED) {
        if (ncol > 0) {
            const f32x4* p = reinterpret_cast<const f32x4*>(base + idx);
            const f32x4 a = p[0], b = p[1];
            x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
            x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = 0.f;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = e < ncol ? base[idx + e] : 0.f;
    }
}

template <bool ALIGNED>
__device__ __forceinline__ void store_f32x8(float* base, int64_t idx, int ncol, const float (&x)[8])
{
    if constexpr (ALIGNED) {
        if (ncol > 0) {
            f32x4* p = reinterpret_cast<f32x4*>(base + idx);
            f32x4 a, b;
            a.x = x[0]; a.y = x[1]; a.z = x[2]; a.w = x[3];
            b.x = x[4]; b.y = x[5]; b.z = x[6]; b.w = x[7];
            p[0] = a;
            p[1] = b;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < ncol) base[idx + e] = x[e];
    }
}

// ---------------------------------------------------------------- reductions

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Sum over the 256 threads of a workgroup, same value returned to every thread.
// Fixed tree, hence deterministic.  lds4: 4 doubles of LDS, reusable afterwards.
__device__ __forceinline__ double block_sum(double v, double* lds4)
{
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) lds4[threadIdx.x >> 6] = v;
    __syncthreads();
    const double total = (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
    __syncthreads();
    return total;
}

struct TileGeom {
    int lane, wave;
    int64_t row0;
    int nrows;
    int64_t col;  // first column of this lane
    int ncol;     // valid columns of this lane: 0..8
};

__device__ __forceinline__ TileGeom tile_geom(const TensorMeta& tm, const WorkItem& it)
{
    TileGeom t;
    t.lane = threadIdx.x & 63;
    t.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    t.row0 = static_cast<int64_t>(it.rb) * tm.tile_rows;
    const int64_t left = tm.n - t.row0;
    t.nrows = static_cast<int>(left < tm.tile_rows ? left : tm.tile_rows);
    t.col = static_cast<int64_t>(it.cb) * kTileCols + t.lane * kLaneCols;
    const int64_t cleft = tm.m - t.col;
    t.ncol = cleft >= kLaneCols ? kLaneCols : (cleft > 0 ? static_cast<int>(cleft) : 0);
    return t;
}

// ---------------------------------------------------------------- vectors

// Algorithm 2 on a 1-D parameter (n x 1 special case: v = r, s = R).  One
// workgroup owns the whole vector; the RMS of Eq. 1 is a workgroup reduction.
template <bool BF16>
__device__ void vector_update(const TensorMeta& tm, const void* g, float* theta, float* state,
                              const SweepHyper& h, const FinalizeHyper& fh, TensorScalars* sc,
                              double* lds4)
{
    float* M = state + tm.off_M;
    float* v = state + tm.off_r;
    float* s = state + tm.off_R;
    const int64_t n = tm.n;
    double acc = 0.0;
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
    for (int64_t i = threadIdx.x; i < n; i += kWorkgroup) {
        const float gi = load_grad1<BF16>(g, i);
        const float uh = kappa * (gi * rsqrtf(v[i]));
        const float Mi = fmaf(h.beta1, M[i], h.one_minus_beta1 * uh);
        M[i] = Mi;
        if (h.algo == CAME_ALGO_CAME) {
            const float dU = uh - Mi;
            const float si = h.beta3 * s[i] + h.one_minus_beta3 * (dU * dU + h.eps2);
            s[i] = si;
            theta[i] = theta[i] - h.lr * Mi * rsqrtf(si);
        } else {
            theta[i] = theta[i] - h.lr * Mi;
        }
    }
}

// ---------------------------------------------------------------- sweep 1

constexpr int kUnroll1 = 4;

template <bool BF16, bool ALIGNED>
__device__ void sweep1_tile(const TensorMeta& tm, const WorkItem& it, const void* g, char* scratch,
                            float* lds /* [4][512] */)
{
    const TileGeom t = tile_geom(tm, it);
    float* rowpart = reinterpret_cast<float*>(scratch + tm.off_rowpart);
    float* colpart = reinterpret_cast<float*>(scratch + tm.off_colpart);
    const int64_t m = tm.m;

    float cacc[kUnroll1][8];
#pragma unroll
    for (int u = 0; u < kUnroll1; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) cacc[u][e] = 0.f;

    for (int i = t.wave; i < t.nrows; i += kWaves * kUnroll1) {
        float x[kUnroll1][8];
#pragma unroll
        for (int u = 0; u < kUnroll1; ++u) {
            const int ii = i + kWaves * u;
            load_grad8<BF16, ALIGNED>(g, (t.row0 + ii) * m + t.col, ii < t.nrows ? t.ncol : 0, x[u]);
        }
#pragma unroll
        for (int u = 0; u < kUnroll1; ++u) {
            const int ii = i + kWaves * u;
            float racc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float sq = x[u][e] * x[u][e];
                racc += sq;
                cacc[u][e] += sq;
            }
            racc = wave_sum(racc);
            if (t.lane == 0 && ii < t.nrows) rowpart[(t.row0 + ii) * tm.CB + it.cb] = racc;
        }
    }

    // column sums of the tile: across the unrolled accumulators, then across the 4 waves
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float v = (cacc[0][e] + cacc[1][e]) + (cacc[2][e] + cacc[3][e]);
        lds[t.wave * kTileCols + t.lane * kLaneCols + e] = v;
    }
    __syncthreads();
    for (int j = threadIdx.x; j < kTileCols; j += kWorkgroup) {
        const int64_t cj = static_cast<int64_t>(it.cb) * kTileCols + j;
        if (cj < m) {
            const float v = (lds[j] + lds[kTileCols + j]) + (lds[2 * kTileCols + j] + lds[3 * kTileCols + j]);
            colpart[static_cast<int64_t>(it.rb) * m + cj] = v;
        }
    }
}

__global__ __launch_bounds__(kWorkgroup) void sweep1_kernel(DeviceTables tb, int32_t item_begin,
                                                            SweepHyper h, FinalizeHyper fh)
{
    __shared__ float lds[kWaves * kTileCols];
    __shared__ double lds4[4];
    const WorkItem it = tb.items[item_begin + blockIdx.x];
    const TensorMeta& tm = tb.metas[it.tensor];
    const void* g = tb.grad[it.tensor];
    const bool bf16 = tm.flags & kFlagBf16Grad;
    if (it.kind == 1) {
        float* theta = static_cast<float*>(tb.theta[it.tensor]);
        if (bf16) vector_update<true>(tm, g, theta, tb.state, h, fh, tb.scalars + it.tensor, lds4);
        else      vector_update<false>(tm, g, theta, tb.state, h, fh, tb.scalars + it.tensor, lds4);
        return;
    }
    const bool aligned = tm.flags & kFlagAligned;
    if (bf16) {
        if (aligned) sweep1_tile<true, true>(tm, it, g, tb.scratch, lds);
        else         sweep1_tile<true, false>(tm, it, g, tb.scratch, lds);
    } else {
        if (aligned) sweep1_tile<false, true>(tm, it, g, tb.scratch, lds);
        else         sweep1_tile<false, false>(tm, it, g, tb.scratch, lds);
    }
}

// ---------------------------------------------------------------- finalize 1

// r_t = beta2 r_{t-1} + (1-beta2)(rowsum g^2 + m eps1), c_t likewise with n eps1
// (eps1 sits inside the sums: m resp. n copies), then sqrt(1^T r_t) by the last
// row workgroup of the tensor to arrive.
__global__ __launch_bounds__(kWorkgroup) void finalize1_kernel(DeviceTables tb, int32_t fin_begin,
                                                               FinalizeHyper h)
{
    __shared__ double lds4[4];
    __shared__ int is_last;
    const FinalizeItem fi = tb.fins[fin_begin + blockIdx.x];
    const TensorMeta& tm = tb.metas[fi.tensor];
    TensorScalars* sc = tb.scalars + fi.tensor;
    const int64_t idx = static_cast<int64_t>(fi.chunk) * kWorkgroup + threadIdx.x;
    if (fi.kind == 0) {
        const float* rowpart = reinterpret_cast<const float*>(tb.scratch + tm.off_rowpart);
        float* r = tb.state + tm.off_r;
        double mine = 0.0;
        if (idx < tm.n) {
            double s = 0.0;
            for (int cb = 0; cb < tm.CB; ++cb) s += static_cast<double>(rowpart[idx * tm.CB + cb]);
            s += static_cast<double>(tm.m) * h.eps1;
            const float rn = static_cast<float>(h.beta2 * static_cast<double>(r[idx]) + h.one_minus_beta2 * s);
            r[idx] = rn;
            mine = static_cast<double>(rn);
        }
        const double total = block_sum(mine, lds4);
        double* fpart = reinterpret_cast<double*>(tb.scratch + tm.off_fpart);
        if (threadIdx.x == 0) {
            fpart[fi.chunk] = total;
            __threadfence();
            const uint32_t prev = atomicAdd(&sc->count_f1, 1u);
            is_last = (prev == static_cast<uint32_t>(tm.f_row_wgs - 1));
        }
        __syncthreads();
        if (is_last) {
            __threadfence();
            double s = 0.0;
            for (int k = threadIdx.x; k < tm.f_row_wgs; k += kWorkgroup)
                s += __hip_atomic_load(&fpart[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s = block_sum(s, lds4);
            if (threadIdx.x == 0) {
                sc->sqrt_sum_r = static_cast<float>(sqrt(s));
                sc->count_f1 = 0u;
            }
        }
    } else {
        const float* colpart = reinterpret_cast<const float*>(tb.scratch + tm.off_colpart);
        float* c = tb.state + tm.off_c;
        if (idx < tm.m) {
            double s = 0.0;
            for (int rb = 0; rb < tm.RB; ++rb) s += static_cast<double>(colpart[static_cast<int64_t>(rb) * tm.m + idx]);
            s += static_cast<double>(tm.n) * h.eps1;
            c[idx] = static_cast<float>(h.beta2 * static_cast<double>(c[idx]) + h.one_minus_beta2 * s);
        }
    }
}

// ---------------------------------------------------------------- sweep 2

constexpr int kUnroll2 = 2;

template <bool BF16, bool ALIGNED>
__device__ void sweep2_tile(const TensorMeta& tm, const WorkItem& it, const void* g, const float* state,
                            char* scratch, const TensorScalars* sc, double* lds /* [4][512] */,
                            double* lds4)
{
    const TileGeom t = tile_geom(tm, it);
    const int64_t m = tm.m;
    const float* r = state + tm.off_r;
    const float* c = state + tm.off_c;
    const float* M = state + tm.off_M;
    double* rowpart = reinterpret_cast<double*>(scratch + tm.off_rowpart);
    double* colpart = reinterpret_cast<double*>(scratch + tm.off_colpart);
    double* tileP = reinterpret_cast<double*>(scratch + tm.off_tileP);
    const float sqrt_sum_r = sc->sqrt_sum_r;

    float b[8];  // rsqrt(c_j) of this lane's columns
#pragma unroll
    for (int e = 0; e < 8; ++e) b[e] = e < t.ncol ? rsqrtf(c[t.col + e]) : 0.f;

    double cP[8], cQ[8], cW[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cP[e] = cQ[e] = cW[e] = 0.0;
    double waveP = 0.0;

    for (int i = t.wave; i < t.nrows; i += kWaves * kUnroll2) {
        float x[kUnroll2][8], mo[kUnroll2][8];
#pragma unroll
        for (int u = 0; u < kUnroll2; ++u) {
            const int ii = i + kWaves * u;
            const int nc = ii < t.nrows ? t.ncol : 0;
            load_grad8<BF16, ALIGNED>(g, (t.row0 + ii) * m + t.col, nc, x[u]);
            load_f32x8<ALIGNED>(M, (t.row0 + ii) * m + t.col, nc, mo[u]);
        }
#pragma unroll
        for (int u = 0; u < kUnroll2; ++u) {
            const int ii = i + kWaves * u;
            if (ii < t.nrows) {
                const float a = rsqrtf(r[t.row0 + ii]) * sqrt_sum_r;  // rsqrt(r_i / 1^T r)
                double rP = 0.0, rQ = 0.0, rW = 0.0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float uf = (x[u][e] * a) * b[e];  // u_ij = g_ij / sqrt(v_ij)
                    const double du = static_cast<double>(uf);
                    const double dm = static_cast<double>(mo[u][e]);
                    rP = fma(du, du, rP); rQ = fma(du, dm, rQ); rW = fma(dm, dm, rW);
                    cP[e] = fma(du, du, cP[e]); cQ[e] = fma(du, dm, cQ[e]); cW[e] = fma(dm, dm, cW[e]);
                }
                rP = wave_sum(rP); rQ = wave_sum(rQ); rW = wave_sum(rW);
                if (t.lane == 0) {
                    double* dst = rowpart + ((t.row0 + ii) * tm.CB + it.cb) * 3;
                    dst[0] = rP; dst[1] = rQ; dst[2] = rW;
                }
                waveP += rP;
            }
        }
    }

    // column sums across the 4 waves, one statistic at a time through 16 KB of LDS
#pragma unroll
    for (int q = 0; q < 3; ++q) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            lds[t.wave * kTileCols + t.lane * kLaneCols + e] = q == 0 ? cP[e] : (q == 1 ? cQ[e] : cW[e]);
        __syncthreads();
        for (int j = threadIdx.x; j < kTileCols; j += kWorkgroup) {
            const int64_t cj = static_cast<int64_t>(it.cb) * kTileCols + j;
            if (cj < m) {
                const double v = (lds[j] + lds[kTileCols + j]) + (lds[2 * kTileCols + j] + lds[3 * kTileCols + j]);
                colpart[(static_cast<int64_t>(it.rb) * 3 + q) * m + cj] = v;
            }
        }
        __syncthreads();
    }
    // sum of u^2 over the tile (feeds RMS(u_t))
    if (t.lane == 0) lds4[t.wave] = waveP;
    __syncthreads();
    if (threadIdx.x == 0)
        tileP[static_cast<int64_t>(it.rb) * tm.CB + it.cb] = (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
}

__global__ __launch_bounds__(kWorkgroup) void sweep2_kernel(DeviceTables tb, int32_t item_begin, SweepHyper h)
{
    __shared__ double lds[kWaves * kTileCols];
    __shared__ double lds4[4];
    (void)h;
    const WorkItem it = tb.items[item_begin + blockIdx.x];
    const TensorMeta& tm = tb.metas[it.tensor];
    const void* g = tb.grad[it.tensor];
    const TensorScalars* sc = tb.scalars + it.tensor;
    const bool bf16 = tm.flags & kFlagBf16Grad;
    const bool aligned = tm.flags & kFlagAligned;
    if (bf16) {
        if (aligned) sweep2_tile<true, true>(tm, it, g, tb.state, tb.scratch, sc, lds, lds4);
        else         sweep2_tile<true, false>(tm, it, g, tb.state, tb.scratch, sc, lds, lds4);
    } else {
        if (aligned) sweep2_tile<false, true>(tm, it, g, tb.state, tb.scratch, sc, lds, lds4);
        else         sweep2_tile<false, false>(tm, it, g, tb.state, tb.scratch, sc, lds, lds4);
    }
}

// ---------------------------------------------------------------- finalize 2

// kappa from the per-tile sums of u^2 (Eq. 1), then
//   rowsum U_i = beta1^2 (kappa^2 P_i - 2 kappa Q_i + W_i),
//   R_t = beta3 R_{t-1} + (1-beta3)(rowsum U + m eps2), C_t likewise with n eps2,
// and sqrt(1^T R_t) by the last row workgroup of the tensor to arrive.
__global__ __launch_bounds__(kWorkgroup) void finalize2_kernel(DeviceTables tb, int32_t fin_begin,
                                                               FinalizeHyper h)
{
    __shared__ double lds4[4];
    __shared__ int is_last;
    const FinalizeItem fi = tb.fins[fin_begin + blockIdx.x];
    const TensorMeta& tm = tb.metas[fi.tensor];
    TensorScalars* sc = tb.scalars + fi.tensor;
    const int64_t idx = static_cast<int64_t>(fi.chunk) * kWorkgroup + threadIdx.x;

    // every finalize workgroup of the tensor re-derives kappa from the same list in the
    // same order, so all agree bit for bit and no extra launch is needed
    const double* tileP = reinterpret_cast<const double*>(tb.scratch + tm.off_tileP);
    double p = 0.0;
    for (int k = threadIdx.x; k < tm.ntiles; k += kWorkgroup) p += tileP[k];
    const double P = block_sum(p, lds4);
    const double rms = sqrt(P / (static_cast<double>(tm.n) * static_cast<double>(tm.m)));
    const double kappa = 1.0 / fmax(1.0, rms / h.clip_d);
    if (fi.kind == 0 && fi.chunk == 0 && threadIdx.x == 0) {
        sc->kappa = static_cast<float>(kappa);
        sc->rms_u = static_cast<float>(rms);
    }
    if (h.algo != CAME_ALGO_CAME) return;

    const double b1sq = h.beta1 * h.beta1;
    if (fi.kind == 0) {
        const double* rowpart = reinterpret_cast<const double*>(tb.scratch + tm.off_rowpart);
        float* R = tb.state + tm.off_R;
        double mine = 0.0;
        if (idx < tm.n) {
            double sP = 0.0, sQ = 0.0, sW = 0.0;
            for (int cb = 0; cb < tm.CB; ++cb) {
                const double* src = rowpart + (idx * tm.CB + cb) * 3;
                sP += src[0]; sQ += src[1]; sW += src[2];
            }
            double U = b1sq * ((kappa * kappa * sP - 2.0 * kappa * sQ) + sW);
            U = fmax(U, 0.0);
            U += static_cast<double>(tm.m) * h.eps2;
            const float Rn = static_cast<float>(h.beta3 * static_cast<double>(R[idx]) + h.one_minus_beta3 * U);
            R[idx] = Rn;
            mine = static_cast<double>(Rn);
        }
        const double total = block_sum(mine, lds4);
        double* fpart = reinterpret_cast<double*>(tb.scratch + tm.off_fpart);
        if (threadIdx.x == 0) {
            fpart[fi.chunk] = total;
            __threadfence();
            const uint32_t prev = atomicAdd(&sc->count_f2, 1u);
            is_last = (prev == static_cast<uint32_t>(tm.f_row_wgs - 1));
        }
        __syncthreads();
        if (is_last) {
            __threadfence();
            double s = 0.0;
            for (int k = threadIdx.x; k < tm.f_row_wgs; k += kWorkgroup)
                s += __hip_atomic_load(&fpart[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s = block_sum(s, lds4);
            if (threadIdx.x == 0) {
                sc->sqrt_sum_R = static_cast<float>(sqrt(s));
                sc->count_f2 = 0u;
            }
        }
    } else {
        const double* colpart = reinterpret_cast<const double*>(tb.scratch + tm.off_colpart);
        float* C = tb.state + tm.off_C;
        if (idx < tm.m) {
            double sP = 0.0, sQ = 0.0, sW = 0.0;
            for (int rb = 0; rb < tm.RB; ++rb) {
                const int64_t base = static_cast<int64_t>(rb) * 3 * tm.m + idx;
                sP += colpart[base]; sQ += colpart[base + tm.m]; sW += colpart[base + 2 * tm.m];
            }
            double U = b1sq * ((kappa * kappa * sP - 2.0 * kappa * sQ) + sW);
            U = fmax(U, 0.0);
            U += static_cast<double>(tm.n) * h.eps2;
            C[idx] = static_cast<float>(h.beta3 * static_cast<double>(C[idx]) + h.one_minus_beta3 * U);
        }
    }
}

// ---------------------------------------------------------------- sweep 3

constexpr int kUnroll3 = 2;

// u^ = kappa g / sqrt(v);  M_t = beta1 M_{t-1} + (1-beta1) u^;
// theta_t = theta_{t-1} - eta M_t / sqrt(S_t)      (Algorithm 1: theta_t = theta_{t-1} - eta M_t)
template <bool BF16, bool ALIGNED>
__device__ void sweep3_tile(const TensorMeta& tm, const WorkItem& it, const void* g, float* theta,
                            float* state, const TensorScalars* sc, const SweepHyper& h)
{
    const TileGeom t = tile_geom(tm, it);
    const int64_t m = tm.m;
    const float* r = state + tm.off_r;
    const float* c = state + tm.off_c;
    const float* R = state + tm.off_R;
    const float* C = state + tm.off_C;
    float* M = state + tm.off_M;
    const bool came = h.algo == CAME_ALGO_CAME;
    const float row_scale_u = sc->sqrt_sum_r * sc->kappa;
    const float row_scale_s = came ? sc->sqrt_sum_R * h.lr : h.lr;

    float b[8], B[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        b[e] = e < t.ncol ? rsqrtf(c[t.col + e]) : 0.f;
        B[e] = came ? (e < t.ncol ? rsqrtf(C[t.col + e]) : 0.f) : 1.f;
    }

    for (int i = t.wave; i < t.nrows; i += kWaves * kUnroll3) {
        float x[kUnroll3][8], mo[kUnroll3][8], th[kUnroll3][8];
#pragma unroll
        for (int u = 0; u < kUnroll3; ++u) {
            const int ii = i + kWaves * u;
            const int nc = ii < t.nrows ? t.ncol : 0;
            const int64_t idx = (t.row0 + ii) * m + t.col;
            load_grad8<BF16, ALIGNED>(g, idx, nc, x[u]);
            load_f32x8<ALIGNED>(M, idx, nc, mo[u]);
            load_f32x8<ALIGNED>(theta, idx, nc, th[u]);
        }
#pragma unroll
        for (int u = 0; u < kUnroll3; ++u) {
            const int ii = i + kWaves * u;
            if (ii < t.nrows) {
                const float a = rsqrtf(r[t.row0 + ii]) * row_scale_u;
                const float A = came ? rsqrtf(R[t.row0 + ii]) * row_scale_s : row_scale_s;
                float mn[8], tn[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float uh = (x[u][e] * a) * b[e];
                    mn[e] = fmaf(h.beta1, mo[u][e], h.one_minus_beta1 * uh);
                    tn[e] = th[u][e] - (mn[e] * A) * B[e];
                }
                const int64_t idx = (t.row0 + ii) * m + t.col;
                store_f32x8<ALIGNED>(M, idx, t.ncol, mn);
                store_f32x8<ALIGNED>(theta, idx, t.ncol, tn);
            }
        }
    }
}

__global__ __launch_bounds__(kWorkgroup) void sweep3_kernel(DeviceTables tb, int32_t item_begin, SweepHyper h)
{
    const WorkItem it = tb.items[item_begin + blockIdx.x];
    const TensorMeta& tm = tb.metas[it.tensor];
    const void* g = tb.grad[it.tensor];
    float* theta = static_cast<float*>(tb.theta[it.tensor]);
    const TensorScalars* sc = tb.scalars + it.tensor;
    const bool bf16 = tm.flags & kFlagBf16Grad;
    const bool aligned = tm.flags & kFlagAligned;
    if (bf16) {
        if (aligned) sweep3_tile<true, true>(tm, it, g, theta, tb.state, sc, h);
        else         sweep3_tile<true, false>(tm, it, g, theta, tb.state, sc, h);
    } else {
        if (aligned) sweep3_tile<false, true>(tm, it, g, theta, tb.state, sc, h);
        else         sweep3_tile<false, false>(tm, it, g, theta, tb.state, sc, h);
    }
}

// ---------------------------------------------------------------- fill

__global__ __launch_bounds__(kWorkgroup) void fill_zero_kernel(f32x4* p4, size_t n4, float* tail, size_t ntail)
{
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    const f32x4 z = {0.f, 0.f, 0.f, 0.f};
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n4; i += stride) p4[i] = z;
    if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0.f;
}

}  // namespace

hipError_t launch_fill_zero(float* p, size_t count, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    const size_t n4 = count / 4;
    const size_t ntail = count % 4;
    size_t blocks = (n4 + kWorkgroup - 1) / kWorkgroup;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (blocks == 0) blocks = 1;
    fill_zero_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(kWorkgroup), 0, s>>>(
        reinterpret_cast<f32x4*>(p), n4, p + n4 * 4, ntail);
    return hipGetLastError();
}

hipError_t launch_fill_zero_bytes(void* p, size_t bytes, hipStream_t s)
{
    return launch_fill_zero(static_cast<float*>(p), bytes / sizeof(float), s);
}

hipError_t launch_sweep1(const DeviceTables& t, int32_t item_begin, int32_t item_end,
                         const SweepHyper& h, const FinalizeHyper& fh, hipStream_t s)
{
    if (item_end <= item_begin) return hipSuccess;
    sweep1_kernel<<<dim3(item_end - item_begin), dim3(kWorkgroup), 0, s>>>(t, item_begin, h, fh);
    return hipGetLastError();
}

hipError_t launch_finalize1(const DeviceTables& t, int32_t fin_begin, int32_t fin_end,
                            const FinalizeHyper& h, hipStream_t s)
{
    if (fin_end <= fin_begin) return hipSuccess;
    finalize1_kernel<<<dim3(fin_end - fin_begin), dim3(kWorkgroup), 0, s>>>(t, fin_begin, h);
    return hipGetLastError();
}

hipError_t launch_sweep2(const DeviceTables& t, int32_t item_begin, int32_t tile_end,
                         const SweepHyper& h, hipStream_t s)
{
    if (tile_end <= item_begin) return hipSuccess;
    sweep2_kernel<<<dim3(tile_end - item_begin), dim3(kWorkgroup), 0, s>>>(t, item_begin, h);
    return hipGetLastError();
}

hipError_t launch_finalize2(const DeviceTables& t, int32_t fin_begin, int32_t fin_end,
                            const FinalizeHyper& h, hipStream_t s)
{
    if (fin_end <= fin_begin) return hipSuccess;
    finalize2_kernel<<<dim3(fin_end - fin_begin), dim3(kWorkgroup), 0, s>>>(t, fin_begin, h);
    return hipGetLastError();
}

hipError_t launch_sweep3(const DeviceTables& t, int32_t item_begin, int32_t tile_end,
                         const SweepHyper& h, hipStream_t s)
{
    if (tile_end <= item_begin) return hipSuccess;
    sweep3_kernel<<<dim3(tile_end - item_begin), dim3(kWorkgroup), 0, s>>>(t, item_begin, h);
    return hipGetLastError();
}

}  // namespace came
