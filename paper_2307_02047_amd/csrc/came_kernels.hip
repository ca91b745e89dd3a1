// gfx950 kernels of the CAME step (Algorithm 2 of the CAME paper).
//
// One step is five grouped launches over ALL tensors of a group (the sweeps once per
// kernel variant present: gradient dtype x aligned/unaligned rows x momentum dtype):
//
//   sweep 1    g            -> row/column partial sums of g^2          (r_t, c_t lines)
//   finalize 1 partials     -> r_t, c_t, sqrt(1^T r_t)
//   sweep 2    g, M_{t-1}   -> row/column partial sums of u^2, u M, M^2 with u = g / sqrt(v_t)
//   finalize 2 partials     -> kappa = 1/max(1, RMS(u_t)/d) (Eq. 1), R_t, C_t, sqrt(1^T R_t)
//   sweep 3    g, M, theta  -> M_t, theta_t;
//                              its first workgroups do the complete update of the 1-D
//                              parameters, one workgroup each (a group without matrices
//                              launches them alone; vectors too long for one workgroup
//                              take two extra launches over chunks)
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
// Tile: 4 wave64s sweep the rows of a 512-column stripe (sweeps 1 and 2: tile_rows of them, tall
// tiles, because every tile costs them partial sums and a chain of dependent loads; sweep 3:
// tile_rows3, short tiles of its own, because it forms no sums and short tiles keep what it reads
// and writes at any one time close together); a lane owns 8 columns of the tile (rows 16-byte
// aligned and no overhanging lane: 4l..4l+3 and 256+4l..256+4l+3, see load_pair; otherwise
// 8l..8l+7), wave w takes rows
// w, w+4, ...  Row sums: 8 in-lane adds, then a wave reduction.  Column sums:
// per-lane accumulators down the tile, combined across the 4 waves in LDS and
// written per (row block, column); the finalize kernels add the row blocks.
// No atomics on data: results are bit-reproducible run to run.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "came_device.hpp"
#include "came_kernels.h"

// Whether the gradient loads of sweeps 1, 2, 3 are streaming (non-temporal) loads.
#ifndef CAME_NT1
#define CAME_NT1 true
#endif
#ifndef CAME_NT2
#define CAME_NT2 true
#endif
#ifndef CAME_NT3
#define CAME_NT3 true
#endif

namespace came {
namespace {

// ---------------------------------------------------------------- long vectors

// Long vectors, pass 1 over chunk `chunk`: v_t and this chunk's sum of u^2.
template <bool BF16>
__device__ void vector_pass1(const TensorMeta& tm, int chunk, const void* g, float* state,
                             const SweepHyper& h, char* scratch, double* lds4)
{
    float* v = state + tm.off_r;
    const int64_t lo = static_cast<int64_t>(chunk) * tm.tile_rows;
    const int64_t hi = lo + tm.tile_rows < tm.n ? lo + tm.tile_rows : tm.n;
    double acc = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kWorkgroup) {
        const float gi = load_grad1<BF16>(g, i);
        const float vi = h.beta2 * v[i] + h.one_minus_beta2 * (gi * gi + h.eps1);
        v[i] = vi;
        const float u = gi * rsqrtf(vi);
        acc += static_cast<double>(u) * static_cast<double>(u);
    }
    const double P = block_sum(acc, lds4);
    if (threadIdx.x == 0) reinterpret_cast<double*>(scratch + tm.off_tileP)[chunk] = P;
}

// Long vectors, pass 2: kappa from the chunk sums (every workgroup, same order, same bits),
// then momentum, confidence and parameter of this chunk.
template <bool BF16>
__device__ void vector_pass2(const TensorMeta& tm, int chunk, const void* g, float* theta, uint16_t* theta16, float* state,
                             const SweepHyper& h, const FinalizeHyper& fh, TensorScalars* sc,
                             const char* scratch, double* lds4)
{
    float* M = state + tm.off_M;
    const float* v = state + tm.off_r;
    float* s = state + tm.off_R;
    const bool mb16 = tm.flags & kFlagBf16Momentum;
    const bool came = h.algo == CAME_ALGO_CAME && !(tm.flags & kFlagMomentumOnly);
    const double* part = reinterpret_cast<const double*>(scratch + tm.off_tileP);
    double p = 0.0;
    for (int k = threadIdx.x; k < tm.ntiles; k += kWorkgroup) p += part[k];
    const double P = block_sum(p, lds4);
    const double rms = sqrt(P / static_cast<double>(tm.n));
    const float kappa = static_cast<float>(1.0 / fmax(1.0, rms / fh.clip_d));
    if (chunk == 0 && threadIdx.x == 0) {
        sc->kappa = kappa;
        sc->rms_u = static_cast<float>(rms);
    }
    const int64_t lo = static_cast<int64_t>(chunk) * tm.tile_rows;
    const int64_t hi = lo + tm.tile_rows < tm.n ? lo + tm.tile_rows : tm.n;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kWorkgroup) {
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

// ---------------------------------------------------------------- row scheduling

// Rows of a tile are dealt to the 4 waves round-robin: wave w owns rows w, w+4, ...
// (`cnt` of them).  They are consumed in batches of U rows; while one batch is consumed
// the next batch's loads are in flight (two register buffers).  The loads of the
// pipelined loop sit in straight-line code -- no branch between a load and the wait that
// precedes its use -- so the compiler can wait for exactly the older batch
// (s_waitcnt vmcnt(N)) instead of draining everything.  For that the batch index is
// clamped (the last trip re-requests the batch it already holds: an L2 hit) and, in
// tiles that overhang the matrix on the right, lanes beyond the last column load from
// the tile's first columns and are masked afterwards.  Rows left over after the full
// batches go through a plain one-row loop.
struct WaveRows {
    int cnt;    // rows of the tile owned by this wave
    int nfull;  // full batches among them
};

template <int U>
__device__ __forceinline__ WaveRows wave_rows(const TileGeom& t)
{
    WaveRows w;
    w.cnt = t.wave < t.nrows ? (t.nrows - t.wave + kWaves - 1) / kWaves : 0;
    w.nfull = w.cnt / U;
    return w;
}


// Which work item a workgroup of a sweep launch takes.  The dispatcher deals consecutive
// workgroups round-robin to the 8 XCDs (workgroup b runs on XCD b % 8), each with its own L2
// and translation cache.  Taking items in launch order would spread every 8 neighbouring
// tiles over all XCDs; instead XCD x works through the chunks x, x+8, x+16, ... of kXcdChunk
// consecutive tiles, so that each XCD streams through compact address ranges (measured on the
// Llama-shaped list: sweep 2 3 % faster, sweep 3 1 %; one contiguous eighth per XCD is as good
// there but unbalances short launches).  A bijection on [0, n) whatever the hardware does.
#ifndef CAME_XCD_CHUNK
#define CAME_XCD_CHUNK 64
#endif
constexpr int32_t kXcds = kNumXcds, kXcdChunk = CAME_XCD_CHUNK;

__device__ __forceinline__ int32_t xcd_item(int32_t b, int32_t n)
{
    const int32_t whole = n / (kXcds * kXcdChunk) * (kXcds * kXcdChunk);
    if (b >= whole) return b;  // the launch's ragged end keeps launch order
    const int32_t x = b % kXcds, j = b / kXcds;
    return ((j / kXcdChunk) * kXcds + x) * kXcdChunk + j % kXcdChunk;
}

// ---------------------------------------------------------------- sweep 1

#ifndef CAME_ROWS1
#define CAME_ROWS1 4
#endif
constexpr int kRows1 = CAME_ROWS1;

// ALIGNED: rows start 16-byte aligned (m % 8 == 0).
// SHAPE: kTileFull (the tile's 512 columns all exist), kTileRagged (the matrix ends inside the
// tile), kTileFolded (tile of the ceil(n/2) x 2m view of a folded matrix, t from folded_geom).
//
// Folded tiles.  A matrix of width m = 512 k + 256 is swept as rows of 2m entries, row 2v of the
// matrix followed by row 2v+1 (which is how they lie in memory), cut into 2k+1 column blocks of
// 512: blocks 0..k-1 lie in row 2v, blocks k+1..2k in row 2v+1, and block k straddles (its first
// 256 columns are the last 256 of row 2v, its last 256 the first 256 of row 2v+1).  Folded tiles
// have 16-byte aligned rows and no overhanging lanes, so they always run with split ownership
// (see load_pair): a lane's first group of 4 columns lies in the tile's first half, its second
// group in the second half, and in the straddling block therefore in the pair's first and second
// row -- for every lane alike.  The sums go where the finalize kernels expect them: column
// partials as if the two rows of a pair belonged to two row blocks (2 rb and 2 rb + 1), row
// partials in slot (column block - k * [row is odd]), which numbers the k+1 blocks that touch a
// row 0..k for even and odd rows alike.
enum TileShape : int { kTileFull = 0, kTileRagged = 1, kTileFolded = 2 };

// What a folded tile adds to the geometry (all trivial for the other shapes).
struct FoldInfo {
    int64_t pitch;   // elements from one row of the tile to the next: 2m (folded) or m
    int64_t mrow0;   // first row of the matrix in the tile
    int mrows;       // rows of the matrix in the tile
    int k;           // index of the straddling column block
    bool split;      // this tile is the straddling one
};

template <int SHAPE>
__device__ __forceinline__ FoldInfo fold_info(const TensorMeta& tm, const WorkItem& it, const TileGeom& t)
{
    FoldInfo f;
    if constexpr (SHAPE == kTileFolded) {
        f.pitch = 2 * tm.m;
        f.mrow0 = 2 * t.row0;
        const int64_t left = tm.n - f.mrow0;
        f.mrows = static_cast<int>(left < 2 * t.nrows ? left : 2 * t.nrows);
        f.k = static_cast<int>(tm.m / kTileCols);
        f.split = it.cb == f.k;
    } else {
        f.pitch = tm.m; f.mrow0 = t.row0; f.mrows = t.nrows; f.k = 0; f.split = false;
    }
    return f;
}

template <bool BF16, bool ALIGNED, int SHAPE>
__device__ void sweep1_tile(const TensorMeta& tm, const WorkItem& it, const TileGeom& t, const void* g,
                            char* scratch, float* lds /* [4][512] */, float* rowbuf /* [rows of the matrix in a tile] */)
{
    constexpr bool FULL = SHAPE != kTileRagged;
    constexpr bool FOLDED = SHAPE == kTileFolded;
    float* rowpart = reinterpret_cast<float*>(scratch + tm.off_rowpart);
    float* colpart = reinterpret_cast<float*>(scratch + tm.off_colpart);
    const int64_t m = tm.m;
    const bool lane_valid = t.ncol > 0;
    const int64_t lcol = ALIGNED ? load_col<FULL>(t, it.cb) : t.col;
    const int lncol = ALIGNED ? kLaneCols : t.ncol;
    const FoldInfo f = fold_info<SHAPE>(tm, it, t);
    // aligned rows, no overhanging lanes: split ownership (see load_pair)
    constexpr bool SPLIT = ALIGNED && SHAPE != kTileRagged;
    const SplitGeom sg = split_geom<FOLDED>(tm, it, t);

    float cacc[2][8];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) cacc[u][e] = 0.f;

    // real = false: the request of the pipelined loop's last trip, whose data nobody uses (see
    // "row scheduling" above).  Gradient loads are streaming loads that leave nothing in the
    // cache, so asking for the last batch a second time would fetch it from memory a second time
    // (measured: 17 % more bytes fetched by sweep 1 at 80-row tiles); that request reads the
    // tensor's descriptor instead, which every workgroup keeps hot in L2.
    auto load_row = [&](int j, bool real = true) {
        if constexpr (SPLIT) {
            const SplitStep st = split_step<FOLDED>(t, sg, j, f.pitch, f.mrows, m);
            return load_pair<BF16, CAME_NT1>(real ? g : static_cast<const void*>(&tm), real ? st.ia : int64_t(0), real ? st.ib : int64_t(4));
        } else {
            return load_grad_raw<BF16, ALIGNED, CAME_NT1>(real ? g : static_cast<const void*>(&tm),
                                                real ? (t.row0 + t.wave + kWaves * j) * m + lcol : int64_t(0), real ? lncol : kLaneCols);
        }
    };
    auto consume_row = [&](const GradRaw<BF16>& raw, int j, int slot) {
        float x[8];
        unpack<BF16>(raw, x);
        if constexpr (SPLIT) {
            const SplitStep st = split_step<FOLDED>(t, sg, j, f.pitch, f.mrows, m);
            float ra = 0.f, rb = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (FOLDED) x[e] = (e < 4 ? st.oka : st.okb) ? x[e] : 0.f;
                if (e < 4) ra = fmaf(x[e], x[e], ra); else rb = fmaf(x[e], x[e], rb);
                cacc[slot][e] = fmaf(x[e], x[e], cacc[slot][e]);
            }
            if (FOLDED && f.split) {  // the two groups lie in the two rows of the pair
                ra = wave_sum_lane63(ra);
                rb = wave_sum_lane63(rb);
                if (t.lane == 63) {
                    rowbuf[st.rowa] = ra;
                    if (st.okb) rowbuf[st.rowb] = rb;
                }
            } else {
                ra = wave_sum_lane63(ra + rb);
                if (t.lane == 63 && st.oka) rowbuf[st.rowa] = ra;
            }
            return;
        }
        float racc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (ALIGNED && !FULL) x[e] = lane_valid ? x[e] : 0.f;
            racc = fmaf(x[e], x[e], racc);
            cacc[slot][e] = fmaf(x[e], x[e], cacc[slot][e]);
        }
        racc = wave_sum_lane63(racc);
        if (t.lane == 63) rowbuf[t.wave + kWaves * j] = racc;
    };

    const WaveRows wr = wave_rows<kRows1>(t);
    if (wr.nfull > 0) {
        GradRaw<BF16> A[kRows1], B[kRows1];
#pragma unroll
        for (int u = 0; u < kRows1; ++u) A[u] = load_row(u);
        for (int k = 0;; k += 2) {
            const int kb = min(k + 1, wr.nfull - 1);
#pragma unroll
            for (int u = 0; u < kRows1; ++u) B[u] = load_row(kb * kRows1 + u, k + 1 < wr.nfull);
#pragma unroll
            for (int u = 0; u < kRows1; ++u) consume_row(A[u], k * kRows1 + u, u & 1);
            if (k + 1 >= wr.nfull) break;
            const int ka = min(k + 2, wr.nfull - 1);
#pragma unroll
            for (int u = 0; u < kRows1; ++u) A[u] = load_row(ka * kRows1 + u, k + 2 < wr.nfull);
#pragma unroll
            for (int u = 0; u < kRows1; ++u) consume_row(B[u], (k + 1) * kRows1 + u, u & 1);
            if (k + 2 >= wr.nfull) break;
        }
    }
    for (int j = wr.nfull * kRows1; j < wr.cnt; ++j) consume_row(load_row(j), j, 0);

    // column sums of the tile: the two accumulator sets, then the 4 waves through LDS
#pragma unroll
    for (int e = 0; e < 8; ++e)
        lds[t.wave * kTileCols + (SPLIT ? split_slot(t.lane, e) : t.lane * kLaneCols + e)] = cacc[0][e] + cacc[1][e];
    __syncthreads();
    for (int j = threadIdx.x; j < kTileCols; j += kWorkgroup) {
        int64_t cj = static_cast<int64_t>(it.cb) * kTileCols + j;
        int64_t prb = it.rb;
        if constexpr (FOLDED) {  // the pair's second row counts as a row block of its own
            const int second = cj >= m ? 1 : 0;
            cj -= second * m;
            prb = 2 * prb + second;
        }
        if (cj < m) {
            const float v = (lds[j] + lds[kTileCols + j]) + (lds[2 * kTileCols + j] + lds[3 * kTileCols + j]);
            colpart[prb * m + cj] = v;
        }
    }
    // row sums of the tile, coalesced: rowpart[column block][row]
    for (int i = threadIdx.x; i < f.mrows; i += kWorkgroup) {
        if constexpr (FOLDED) {
            const int odd = i & 1;  // (the tile's first row of the matrix is even)
            if (odd ? it.cb >= f.k : it.cb <= f.k)
                rowpart[static_cast<int64_t>(it.cb - odd * f.k) * tm.n + f.mrow0 + i] = rowbuf[i];
        } else {
            rowpart[static_cast<int64_t>(it.cb) * tm.n + f.mrow0 + i] = rowbuf[i];
        }
    }
}

// One __global__ entry per variant, each with the occupancy (waves per SIMD) its register
// budget is tuned for: the compiler keeps the kernel within 512/N VGPRs.
#ifndef CAME_WAVES1
#define CAME_WAVES1 5
#endif
#define CAME_SWEEP1_KERNEL(NAME, BF16, ALIGNED, WAVES)                                              \
    __global__ __launch_bounds__(kWorkgroup) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES)))     \
    void NAME(DeviceTables tb, int32_t item_begin)                                                  \
    {                                                                                               \
        __shared__ __attribute__((aligned(16))) float lds[kWaves * kTileCols];                      \
        extern __shared__ float rowbuf_f32[];                                                       \
        const WorkItem it = tb.items[item_begin + xcd_item(blockIdx.x, gridDim.x)];                 \
        const TensorMeta& tm = tb.metas[it.tensor];                                                 \
        const bool folded = ALIGNED && it.kind == 6;                                                \
        const TileGeom t = folded ? folded_geom(tm, it, tm.tile_rows) : tile_geom(tm, it);          \
        const void* g = tb.grad[it.tensor];                    \
        const bool full = static_cast<int64_t>(it.cb + 1) * kTileCols <= tm.m;                      \
        if (folded)                                                                                 \
            sweep1_tile<BF16, ALIGNED, ALIGNED ? kTileFolded : kTileFull>(tm, it, t, g, tb.scratch, lds, rowbuf_f32); \
        else if (!ALIGNED || full)                                                                  \
            sweep1_tile<BF16, ALIGNED, kTileFull>(tm, it, t, g, tb.scratch, lds, rowbuf_f32);       \
        else                                                                                        \
            sweep1_tile<BF16, ALIGNED, kTileRagged>(tm, it, t, g, tb.scratch, lds, rowbuf_f32);     \
    }
CAME_SWEEP1_KERNEL(sweep1_bf16_kernel, true, true, CAME_WAVES1)
CAME_SWEEP1_KERNEL(sweep1_f32_kernel, false, true, 4)
CAME_SWEEP1_KERNEL(sweep1_bf16_unaligned_kernel, true, false, 4)
CAME_SWEEP1_KERNEL(sweep1_f32_unaligned_kernel, false, false, 4)

__global__ __launch_bounds__(kWorkgroup) void vector_kernel(DeviceTables tb, int32_t item_begin,
                                                            SweepHyper h, FinalizeHyper fh)
{
    __shared__ double lds4[4];
    vector_item(tb, item_begin + blockIdx.x, h, fh, lds4);
}

__global__ __launch_bounds__(kWorkgroup) void long_vector_kernel(DeviceTables tb, int32_t item_begin, int32_t pass,
                                                                 SweepHyper h, FinalizeHyper fh)
{
    __shared__ double lds4[4];
    const WorkItem it = tb.items[item_begin + blockIdx.x];
    const TensorMeta& tm = tb.metas[it.tensor];
    const void* g = tb.grad[it.tensor];
    float* theta = static_cast<float*>(tb.theta[it.tensor]);
    const bool bf16 = tm.flags & kFlagBf16Grad;
    if (pass == 1) {
        if (bf16) vector_pass1<true>(tm, it.rb, g, tb.state, h, tb.scratch, lds4);
        else      vector_pass1<false>(tm, it.rb, g, tb.state, h, tb.scratch, lds4);
    } else {
        uint16_t* theta16 = static_cast<uint16_t*>(tb.theta16[it.tensor]);
        if (bf16) vector_pass2<true>(tm, it.rb, g, theta, theta16, tb.state, h, fh, tb.scalars + it.tensor, tb.scratch, lds4);
        else      vector_pass2<false>(tm, it.rb, g, theta, theta16, tb.state, h, fh, tb.scalars + it.tensor, tb.scratch, lds4);
    }
}

// ---------------------------------------------------------------- finalize 1

// Column workgroup of a finalize launch: lane l of every wave owns column chunk*64 + l,
// wave w adds the row blocks [rb0, rb1), a quarter of them; wave 0 then combines the four
// partial sums in a fixed order.
struct FinalizeCols {
    int lane, wave;
    int64_t col;
    int rb0, rb1;
};

__device__ __forceinline__ FinalizeCols finalize_cols(const TensorMeta& tm, const FinalizeItem& fi)
{
    FinalizeCols f;
    f.lane = threadIdx.x & 63;
    f.wave = threadIdx.x >> 6;
    f.col = static_cast<int64_t>(fi.chunk) * kFinalizeCols + f.lane;
    const int per = (tm.RB + kWaves - 1) / kWaves;
    f.rb0 = min(f.wave * per, tm.RB);
    f.rb1 = min(f.rb0 + per, tm.RB);
    return f;
}

// r_t = beta2 r_{t-1} + (1-beta2)(rowsum g^2 + m eps1), c_t likewise with n eps1
// (eps1 sits inside the sums: m resp. n copies).  Each row workgroup also leaves the
// sum of its 256 new r values; sweep 2 adds those few numbers up to 1^T r_t.
__global__ __launch_bounds__(kWorkgroup) void finalize1_kernel(DeviceTables tb, int32_t fin_begin,
                                                               FinalizeHyper h)
{
    __shared__ double lds4[4];
    __shared__ double colsum[kWaves][kFinalizeCols];
    const FinalizeItem fi = tb.fins[fin_begin + blockIdx.x];
    const TensorMeta& tm = tb.metas[fi.tensor];
    const int64_t idx = static_cast<int64_t>(fi.chunk) * kWorkgroup + threadIdx.x;
    if (fi.kind == 0) {
        const float* rowpart = reinterpret_cast<const float*>(tb.scratch + tm.off_rowpart);
        float* r = tb.state + tm.off_r;
        double mine = 0.0;
        if (idx < tm.n) {
            double s = 0.0;
#pragma unroll 4
            for (int cb = 0; cb < tm.CB; ++cb) s += static_cast<double>(rowpart[static_cast<int64_t>(cb) * tm.n + idx]);
            s += static_cast<double>(tm.m) * h.eps1;
            const float rn = static_cast<float>(h.beta2 * static_cast<double>(r[idx]) + h.one_minus_beta2 * s);
            r[idx] = rn;
            mine = static_cast<double>(rn);
        }
        const double total = block_sum(mine, lds4);
        if (threadIdx.x == 0) reinterpret_cast<double*>(tb.scratch + tm.off_fpart)[fi.chunk] = total;
    } else {
        const float* colpart = reinterpret_cast<const float*>(tb.scratch + tm.off_colpart);
        float* c = tb.state + tm.off_c;
        const FinalizeCols fc = finalize_cols(tm, fi);
        double s = 0.0;
        if (fc.col < tm.m) {
#pragma unroll 8
            for (int rb = fc.rb0; rb < fc.rb1; ++rb) s += static_cast<double>(colpart[static_cast<int64_t>(rb) * tm.m + fc.col]);
        }
        colsum[fc.wave][fc.lane] = s;
        __syncthreads();
        if (fc.wave == 0 && fc.col < tm.m) {
            s = (colsum[0][fc.lane] + colsum[1][fc.lane]) + (colsum[2][fc.lane] + colsum[3][fc.lane]);
            s += static_cast<double>(tm.n) * h.eps1;
            c[fc.col] = static_cast<float>(h.beta2 * static_cast<double>(c[fc.col]) + h.one_minus_beta2 * s);
        }
    }
}

// ---------------------------------------------------------------- sweep 2

#ifndef CAME_ROWS2
#define CAME_ROWS2 2
#endif
constexpr int kRows2 = CAME_ROWS2;

// CAME_STATS: Algorithm 2 needs all three statistics per row and column.  Algorithm 1
// (no instability / confidence lines) needs only the total of u^2 for Eq. 1, so M is not
// read at all and there are no column accumulators.
// MB16: M is stored as bfloat16.
// SHAPE: TileShape, as in sweep 1.  TRL: rows of the matrix a tile can hold (tile_rows, twice that
// when the list has folded matrices): the stride of the three row-sum arrays in LDS.
// NTM: the momentum loads are streaming loads too (lists that are small against the on-package
// cache, see Plan::keep_tail_cached).
template <bool BF16, bool ALIGNED, int SHAPE, bool CAME_STATS, bool MB16, bool NTM>
__device__ void sweep2_tile(const TensorMeta& tm, const WorkItem& it, const TileGeom& t, const void* g,
                            const float* state, char* scratch, TensorScalars* sc,
                            double* lds /* [4][512] */, double* lds4, double* rowbuf /* [3][TRL] */,
                            float* rowfac /* [TRL] */, int TRL)
{
    constexpr bool FULL = SHAPE != kTileRagged;
    constexpr bool FOLDED = SHAPE == kTileFolded;
    const int64_t m = tm.m;
    const float* r = state + tm.off_r;
    const float* c = state + tm.off_c;
    const float* M = state + tm.off_M;
    double* rowpart = reinterpret_cast<double*>(scratch + tm.off_rowpart);
    double* colpart = reinterpret_cast<double*>(scratch + tm.off_colpart);
    double* tileP = reinterpret_cast<double*>(scratch + tm.off_tileP);
    const bool lane_valid = t.ncol > 0;
    const int64_t lcol = ALIGNED ? load_col<FULL>(t, it.cb) : t.col;
    const int lncol = ALIGNED ? kLaneCols : t.ncol;
    const int TR = TRL;
    const FoldInfo f = fold_info<SHAPE>(tm, it, t);
    // aligned rows, no overhanging lanes: split ownership (see load_pair) -- except where both
    // arrays this sweep reads are bfloat16: split ownership would turn their dense 16-byte loads
    // into pairs of 8-byte ones (measured: sweep 2 7 % slower); folded tiles need it all the same
    constexpr bool SPLIT = ALIGNED && SHAPE != kTileRagged && (SHAPE == kTileFolded || !(BF16 && MB16 && CAME_STATS));
    const SplitGeom sg = split_geom<FOLDED>(tm, it, t);

    struct Row { GradRaw<BF16> g; GradRaw<MB16> mo; };
    // real = false: the pipelined loop's last, unused request; the streaming gradient load of it
    // goes to the tensor's descriptor (hot in L2) instead of fetching the last batch again
    auto load_row = [&](int j, bool real = true) {
        Row x;
        if constexpr (SPLIT) {
            const SplitStep st = split_step<FOLDED>(t, sg, j, f.pitch, f.mrows, m);
            x.g = load_pair<BF16, CAME_NT2>(real ? g : static_cast<const void*>(&tm), real ? st.ia : int64_t(0), real ? st.ib : int64_t(4));
            if constexpr (CAME_STATS) x.mo = load_pair<MB16, NTM>(M, st.ia, st.ib);
            return x;
        }
        const int64_t idx = (t.row0 + t.wave + kWaves * j) * m + lcol;
        x.g = load_grad_raw<BF16, ALIGNED, CAME_NT2>(real ? g : static_cast<const void*>(&tm), real ? idx : int64_t(0), real ? lncol : kLaneCols);
        if constexpr (CAME_STATS) x.mo = load_grad_raw<MB16, ALIGNED, NTM>(M, idx, lncol);
        return x;
    };
    // element-wise loads: one row per batch (address registers); folded tiles likewise (their
    // per-lane row bookkeeping costs registers that this kernel does not have to spare)
    constexpr int U = ALIGNED && !FOLDED ? kRows2 : 1;
    const WaveRows wr = wave_rows<U>(t);
    Row A[U], B[U];
    if (wr.nfull > 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) A[u] = load_row(u);
    }

    // 1^T r_t from the per-workgroup sums finalize 1 left (every wave, same order, same bits)
    const double sum_r = wave_sum_list(reinterpret_cast<const double*>(scratch + tm.off_fpart), tm.f_row_wgs);
    const float sqrt_sum_r = static_cast<float>(sqrt(sum_r));
    if (it.rb == 0 && it.cb == 0 && threadIdx.x == 0) sc->sqrt_sum_r = sqrt_sum_r;

    // per-row factor rsqrt(r_i / 1^T r) of the tile's rows, once, into LDS: inside the row
    // loop it is then an LDS broadcast read and no global load has to be waited for there
    for (int i = threadIdx.x; i < f.mrows; i += kWorkgroup) rowfac[i] = rsqrtf(r[f.mrow0 + i]) * sqrt_sum_r;

    float b[8];  // rsqrt(c_j) of this lane's columns
    {
        float cv[8];
        if constexpr (SPLIT) unpack(load_f32_pair(c, sg.ca, sg.cb), cv);
        else unpack(load_f32_raw<ALIGNED>(c, lcol, lncol), cv);
#pragma unroll
        for (int e = 0; e < 8; ++e) b[e] = (SPLIT || e < t.ncol) ? rsqrtf(cv[e]) : 0.f;
    }
    __syncthreads();

    double cP[8], cQ[8], cW[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cP[e] = cQ[e] = cW[e] = 0.0;

    auto consume_row = [&](const Row& row, int j) {
        if constexpr (SPLIT) {
            const SplitStep st = split_step<FOLDED>(t, sg, j, f.pitch, f.mrows, m);
            // rsqrt(r_i / 1^T r) of the two groups' rows (one row unless the tile spans a pair's two rows)
            const float aa = FOLDED ? (st.oka ? rowfac[st.rowa] : 0.f) : rowfac[st.rowa];
            const float ab = FOLDED ? (st.okb ? rowfac[st.rowb] : 0.f) : aa;
            float x[8];
            unpack<BF16>(row.g, x);
            double pa = 0.0, qa = 0.0, wa = 0.0, pb = 0.0, qb = 0.0, wb = 0.0;
            if constexpr (CAME_STATS) {
                float mo[8];
                unpack<MB16>(row.mo, mo);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (FOLDED) {  // a missing row's lanes hold a copy of the row before it
                        x[e] = (e < 4 ? st.oka : st.okb) ? x[e] : 0.f;
                        mo[e] = (e < 4 ? st.oka : st.okb) ? mo[e] : 0.f;
                    }
                    const float uf = (x[e] * (e < 4 ? aa : ab)) * b[e];  // u_ij = g_ij / sqrt(v_ij)
                    const double du = static_cast<double>(uf);
                    const double dm = static_cast<double>(mo[e]);
                    if (e < 4) { pa = fma(du, du, pa); qa = fma(du, dm, qa); wa = fma(dm, dm, wa); }
                    else       { pb = fma(du, du, pb); qb = fma(du, dm, qb); wb = fma(dm, dm, wb); }
                    cP[e] = fma(du, du, cP[e]); cQ[e] = fma(du, dm, cQ[e]); cW[e] = fma(dm, dm, cW[e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (FOLDED) x[e] = (e < 4 ? st.oka : st.okb) ? x[e] : 0.f;
                    const double du = static_cast<double>((x[e] * (e < 4 ? aa : ab)) * b[e]);
                    if (e < 4) pa = fma(du, du, pa); else pb = fma(du, du, pb);
                }
            }
            if (FOLDED && f.split) {  // the two groups lie in the two rows of the pair
                pa = wave_sum_lane63(pa); pb = wave_sum_lane63(pb);
                if constexpr (CAME_STATS) {
                    qa = wave_sum_lane63(qa); wa = wave_sum_lane63(wa);
                    qb = wave_sum_lane63(qb); wb = wave_sum_lane63(wb);
                }
                if (t.lane == 63) {
                    rowbuf[st.rowa] = pa;
                    if (CAME_STATS) { rowbuf[TR + st.rowa] = qa; rowbuf[2 * TR + st.rowa] = wa; }
                    if (st.okb) {
                        rowbuf[st.rowb] = pb;
                        if (CAME_STATS) { rowbuf[TR + st.rowb] = qb; rowbuf[2 * TR + st.rowb] = wb; }
                    }
                }
            } else {
                pa = wave_sum_lane63(pa + pb);
                if constexpr (CAME_STATS) { qa = wave_sum_lane63(qa + qb); wa = wave_sum_lane63(wa + wb); }
                if (t.lane == 63 && st.oka) {
                    rowbuf[st.rowa] = pa;
                    if (CAME_STATS) { rowbuf[TR + st.rowa] = qa; rowbuf[2 * TR + st.rowa] = wa; }
                }
            }
            return;
        }
        const int i = t.wave + kWaves * j;
        const float a = rowfac[i];  // rsqrt(r_i / 1^T r)
        float x[8];
        unpack<BF16>(row.g, x);
        if constexpr (CAME_STATS) {
            float mo[8];
            unpack<MB16>(row.mo, mo);
            double rP = 0.0, rQ = 0.0, rW = 0.0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (ALIGNED && !FULL) mo[e] = lane_valid ? mo[e] : 0.f;   // (b[e] = 0 already zeroes u)
                const float uf = (x[e] * a) * b[e];  // u_ij = g_ij / sqrt(v_ij)
                const double du = static_cast<double>(uf);
                const double dm = static_cast<double>(mo[e]);
                rP = fma(du, du, rP); rQ = fma(du, dm, rQ); rW = fma(dm, dm, rW);
                cP[e] = fma(du, du, cP[e]); cQ[e] = fma(du, dm, cQ[e]); cW[e] = fma(dm, dm, cW[e]);
            }
            rP = wave_sum_lane63(rP); rQ = wave_sum_lane63(rQ); rW = wave_sum_lane63(rW);
            if (t.lane == 63) { rowbuf[i] = rP; rowbuf[TR + i] = rQ; rowbuf[2 * TR + i] = rW; }
        } else {
            double rP = 0.0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const double du = static_cast<double>((x[e] * a) * b[e]);
                rP = fma(du, du, rP);
            }
            rP = wave_sum_lane63(rP);
            if (t.lane == 63) rowbuf[i] = rP;
        }
    };

    if (wr.nfull > 0) {
        for (int k = 0;; k += 2) {
            const int kb = min(k + 1, wr.nfull - 1);
#pragma unroll
            for (int u = 0; u < U; ++u) B[u] = load_row(kb * U + u, k + 1 < wr.nfull);
#pragma unroll
            for (int u = 0; u < U; ++u) consume_row(A[u], k * U + u);
            if (k + 1 >= wr.nfull) break;
            const int ka = min(k + 2, wr.nfull - 1);
#pragma unroll
            for (int u = 0; u < U; ++u) A[u] = load_row(ka * U + u, k + 2 < wr.nfull);
#pragma unroll
            for (int u = 0; u < U; ++u) consume_row(B[u], (k + 1) * U + u);
            if (k + 2 >= wr.nfull) break;
        }
    }
    for (int j = wr.nfull * U; j < wr.cnt; ++j) consume_row(load_row(j), j);

    // column sums across the 4 waves, one statistic at a time through 16 KB of LDS
    if constexpr (!CAME_STATS) __syncthreads();
#pragma unroll
    for (int q = 0; q < (CAME_STATS ? 3 : 0); ++q) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            lds[t.wave * kTileCols + (SPLIT ? split_slot(t.lane, e) : t.lane * kLaneCols + e)] = q == 0 ? cP[e] : (q == 1 ? cQ[e] : cW[e]);
        __syncthreads();
        for (int j = threadIdx.x; j < kTileCols; j += kWorkgroup) {
            int64_t cj = static_cast<int64_t>(it.cb) * kTileCols + j;
            int64_t prb = it.rb;
            if constexpr (FOLDED) {  // the pair's second row counts as a row block of its own
                const int second = cj >= m ? 1 : 0;
                cj -= second * m;
                prb = 2 * prb + second;
            }
            if (cj < m) {
                const double v = (lds[j] + lds[kTileCols + j]) + (lds[2 * kTileCols + j] + lds[3 * kTileCols + j]);
                colpart[(prb * 3 + q) * m + cj] = v;
            }
        }
        __syncthreads();
    }
    // row sums of the tile, coalesced: rowpart[column block][statistic][row]; and the
    // tile's sum of u^2 (feeds RMS(u_t))
    double p = 0.0;
    for (int i = threadIdx.x; i < f.mrows; i += kWorkgroup) {
        int slot = it.cb;
        if constexpr (FOLDED) {
            const int odd = i & 1;  // (the tile's first row of the matrix is even)
            if (!(odd ? it.cb >= f.k : it.cb <= f.k)) continue;  // a row this tile has no entry of
            slot = it.cb - odd * f.k;
        }
        const double vP = rowbuf[i];
        p += vP;
        if constexpr (CAME_STATS) {
            const int64_t base = static_cast<int64_t>(slot) * 3 * tm.n + f.mrow0 + i;
            rowpart[base] = vP;
            rowpart[base + tm.n] = rowbuf[TR + i];
            rowpart[base + 2 * tm.n] = rowbuf[2 * TR + i];
        }
    }
    p = block_sum(p, lds4);
    if (threadIdx.x == 0) tileP[static_cast<int64_t>(it.rb) * (FOLDED ? 2 * f.k + 1 : tm.CB) + it.cb] = p;
}

#ifndef CAME_WAVES2
#define CAME_WAVES2 3
#endif
#define CAME_SWEEP2_KERNEL(NAME, BF16, ALIGNED, STATS, MB16, WAVES, NTM)                                             \
    __global__ __launch_bounds__(kWorkgroup) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES)))     \
    void NAME(DeviceTables tb, int32_t item_begin, int32_t reverse, int32_t lds_rows)               \
    {                                                                                               \
        __shared__ double lds[kWaves * kTileCols];                                                  \
        __shared__ double lds4[4];                                                                  \
        extern __shared__ double rowbuf_f64[];                                                      \
        const int32_t ord = xcd_item(blockIdx.x, gridDim.x);                                        \
        const WorkItem it = tb.items[item_begin + (reverse ? static_cast<int32_t>(gridDim.x) - 1 - ord : ord)]; \
        const TensorMeta& tm = tb.metas[it.tensor];                                                 \
        const bool folded = ALIGNED && it.kind == 6;                                                \
        const TileGeom t = folded ? folded_geom(tm, it, tm.tile_rows) : tile_geom(tm, it);          \
        float* rowfac = reinterpret_cast<float*>(rowbuf_f64 + 3 * lds_rows);                        \
        const void* g = tb.grad[it.tensor];                    \
        const bool full = static_cast<int64_t>(it.cb + 1) * kTileCols <= tm.m;                      \
        if (folded)                                                                                 \
            sweep2_tile<BF16, ALIGNED, ALIGNED ? kTileFolded : kTileFull, STATS, MB16, NTM>(tm, it, t, g, tb.state, tb.scratch, \
                                             tb.scalars + it.tensor, lds, lds4, rowbuf_f64, rowfac, lds_rows); \
        else if (!ALIGNED || full)                                                                  \
            sweep2_tile<BF16, ALIGNED, kTileFull, STATS, MB16, NTM>(tm, it, t, g, tb.state, tb.scratch,  \
                                             tb.scalars + it.tensor, lds, lds4, rowbuf_f64, rowfac, lds_rows); \
        else                                                                                        \
            sweep2_tile<BF16, ALIGNED, kTileRagged, STATS, MB16, NTM>(tm, it, t, g, tb.state, tb.scratch, \
                                              tb.scalars + it.tensor, lds, lds4, rowbuf_f64, rowfac, lds_rows); \
    }
CAME_SWEEP2_KERNEL(sweep2_bf16_kernel, true, true, true, false, CAME_WAVES2, false)
CAME_SWEEP2_KERNEL(sweep2_f32_kernel, false, true, true, false, 2, false)
CAME_SWEEP2_KERNEL(sweep2_bf16_unaligned_kernel, true, false, true, false, 3, false)
CAME_SWEEP2_KERNEL(sweep2_f32_unaligned_kernel, false, false, true, false, 3, false)
CAME_SWEEP2_KERNEL(sweep2_bf16_mbf16_kernel, true, true, true, true, CAME_WAVES2, false)
CAME_SWEEP2_KERNEL(sweep2_f32_mbf16_kernel, false, true, true, true, 2, false)
CAME_SWEEP2_KERNEL(sweep2_bf16_mbf16_unaligned_kernel, true, false, true, true, 3, false)
CAME_SWEEP2_KERNEL(sweep2_f32_mbf16_unaligned_kernel, false, false, true, true, 3, false)
CAME_SWEEP2_KERNEL(sweep2_bf16_ntm_kernel, true, true, true, false, CAME_WAVES2, true)
CAME_SWEEP2_KERNEL(sweep2_f32_ntm_kernel, false, true, true, false, 2, true)
CAME_SWEEP2_KERNEL(sweep2_bf16_mbf16_ntm_kernel, true, true, true, true, CAME_WAVES2, true)
CAME_SWEEP2_KERNEL(sweep2_f32_mbf16_ntm_kernel, false, true, true, true, 2, true)
// Algorithm 1: M is not read, so its storage type does not matter here
CAME_SWEEP2_KERNEL(sweep2_adafactor_bf16_kernel, true, true, false, false, 8, false)
CAME_SWEEP2_KERNEL(sweep2_adafactor_f32_kernel, false, true, false, false, 8, false)
CAME_SWEEP2_KERNEL(sweep2_adafactor_bf16_unaligned_kernel, true, false, false, false, 4, false)
CAME_SWEEP2_KERNEL(sweep2_adafactor_f32_unaligned_kernel, false, false, false, false, 4, false)

// ---------------------------------------------------------------- finalize 2

// kappa from the per-tile sums of u^2 (Eq. 1), then
//   rowsum U_i = beta1^2 (kappa^2 P_i - 2 kappa Q_i + W_i),
//   R_t = beta3 R_{t-1} + (1-beta3)(rowsum U + m eps2), C_t likewise with n eps2.
// Each row workgroup also leaves the sum of its 256 new R values; sweep 3 adds those
// few numbers up to 1^T R_t.
__global__ __launch_bounds__(kWorkgroup) void finalize2_kernel(DeviceTables tb, int32_t fin_begin,
                                                               FinalizeHyper h)
{
    __shared__ double lds4[4];
    __shared__ double colsum[3][kWaves][kFinalizeCols];
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
    const double k2 = kappa * kappa, km2 = -2.0 * kappa;
    if (fi.kind == 0) {
        const double* rowpart = reinterpret_cast<const double*>(tb.scratch + tm.off_rowpart);
        float* R = tb.state + tm.off_R;
        double mine = 0.0;
        if (idx < tm.n) {
            double sP = 0.0, sQ = 0.0, sW = 0.0;
#pragma unroll 4
            for (int cb = 0; cb < tm.CB; ++cb) {
                const int64_t base = static_cast<int64_t>(cb) * 3 * tm.n + idx;
                sP += rowpart[base]; sQ += rowpart[base + tm.n]; sW += rowpart[base + 2 * tm.n];
            }
            double U = b1sq * ((k2 * sP + km2 * sQ) + sW);
            U = U < 0.0 ? 0.0 : U;  // rounding of the three-term sum; a NaN stays a NaN
            U += static_cast<double>(tm.m) * h.eps2;
            const float Rn = static_cast<float>(h.beta3 * static_cast<double>(R[idx]) + h.one_minus_beta3 * U);
            R[idx] = Rn;
            mine = static_cast<double>(Rn);
        }
        const double total = block_sum(mine, lds4);
        if (threadIdx.x == 0)
            reinterpret_cast<double*>(tb.scratch + tm.off_fpart)[tm.f_row_wgs + fi.chunk] = total;
    } else {
        const double* colpart = reinterpret_cast<const double*>(tb.scratch + tm.off_colpart);
        float* C = tb.state + tm.off_C;
        const FinalizeCols fc = finalize_cols(tm, fi);
        double sP = 0.0, sQ = 0.0, sW = 0.0;
        if (fc.col < tm.m) {
#pragma unroll 4
            for (int rb = fc.rb0; rb < fc.rb1; ++rb) {
                const int64_t base = static_cast<int64_t>(rb) * 3 * tm.m + fc.col;
                sP += colpart[base]; sQ += colpart[base + tm.m]; sW += colpart[base + 2 * tm.m];
            }
        }
        colsum[0][fc.wave][fc.lane] = sP; colsum[1][fc.wave][fc.lane] = sQ; colsum[2][fc.wave][fc.lane] = sW;
        __syncthreads();
        if (fc.wave == 0 && fc.col < tm.m) {
            const int l = fc.lane;
            sP = (colsum[0][0][l] + colsum[0][1][l]) + (colsum[0][2][l] + colsum[0][3][l]);
            sQ = (colsum[1][0][l] + colsum[1][1][l]) + (colsum[1][2][l] + colsum[1][3][l]);
            sW = (colsum[2][0][l] + colsum[2][1][l]) + (colsum[2][2][l] + colsum[2][3][l]);
            double U = b1sq * ((k2 * sP + km2 * sQ) + sW);
            U = U < 0.0 ? 0.0 : U;  // rounding of the three-term sum; a NaN stays a NaN
            U += static_cast<double>(tm.n) * h.eps2;
            C[fc.col] = static_cast<float>(h.beta3 * static_cast<double>(C[fc.col]) + h.one_minus_beta3 * U);
        }
    }
}

// ---------------------------------------------------------------- sweep 3

#ifndef CAME_ROWS3
#define CAME_ROWS3 1
#endif
constexpr int kRows3 = CAME_ROWS3;

// u^ = kappa g / sqrt(v);  M_t = beta1 M_{t-1} + (1-beta1) u^;
// theta_t = theta_{t-1} - eta M_t / sqrt(S_t)      (Algorithm 1: theta_t = theta_{t-1} - eta M_t);
// with a decoupled weight decay theta_{t-1} is first scaled by h.decay = 1 - eta lambda.
// COPY16: also write theta_t as bfloat16 to theta16 (came_step_bf16_copy).
// MB16: M is stored as bfloat16; theta_t is formed from the unrounded M_t.
// SHAPE: kTileFull (the tile's 512 columns exist), kTileRagged (the matrix ends inside the
// tile), kTileFolded (tile of the ceil(n/2) x 2m view of a folded matrix, t from folded_geom: a
// step of the wave covers 512 consecutive entries of rows 2v, 2v+1 as they lie in memory, each
// lane with the row and column factors of the entry it really holds).
template <bool BF16, bool ALIGNED, int SHAPE, bool COPY16, bool MB16>
__device__ void sweep3_tile(const TensorMeta& tm, const WorkItem& it, const TileGeom& t, const void* g,
                            float* theta, void* theta16, float* state, const char* scratch,
                            const TensorScalars* sc, const SweepHyper& h, float* rowfac /* [2][2 tile_rows3] */)
{
    constexpr bool FULL = SHAPE != kTileRagged;
    constexpr bool FOLDED = SHAPE == kTileFolded;
    const int64_t m = tm.m;
    const int64_t pitch = FOLDED ? 2 * m : m;  // elements from one row of the tile to the next
    const int TR = 2 * tm.tile_rows3;           // room per factor array: a folded tile has two rows of the matrix per row
    const float* r = state + tm.off_r;
    const float* c = state + tm.off_c;
    const float* R = state + tm.off_R;
    const float* C = state + tm.off_C;
    float* M = state + tm.off_M;
    const bool came = h.algo == CAME_ALGO_CAME;
    const int64_t lcol = ALIGNED ? load_col<FULL>(t, it.cb) : t.col;
    const int lncol = ALIGNED ? kLaneCols : t.ncol;
    // folded tiles: rows of the matrix in the tile, first of them, this lane's column in the matrix
    const int64_t mrow0 = FOLDED ? 2 * t.row0 : t.row0;
    const int mrows = FOLDED ? static_cast<int>(min(static_cast<int64_t>(2 * t.nrows), tm.n - mrow0)) : t.nrows;
    // aligned rows, no overhanging lanes: split ownership (see load_pair)
    constexpr bool SPLIT = ALIGNED && SHAPE != kTileRagged;
    const SplitGeom sg = split_geom<FOLDED>(tm, it, t);

    struct Row { GradRaw<BF16> g; GradRaw<MB16> mo; F32Raw th; };
    // real = false: the pipelined loop's last, unused request; the streaming gradient load of it
    // goes to the tensor's descriptor (hot in L2) instead of fetching the last batch again
    auto load_row = [&](int j, bool real = true) {
        Row x;
        if constexpr (SPLIT) {
            const SplitStep st = split_step<FOLDED>(t, sg, j, pitch, mrows, m);
            x.g = load_pair<BF16, CAME_NT3>(real ? g : static_cast<const void*>(&tm), real ? st.ia : int64_t(0), real ? st.ib : int64_t(4));
            x.mo = load_pair<MB16, false>(M, st.ia, st.ib);
            x.th = load_f32_pair(theta, st.ia, st.ib);
            return x;
        }
        const int64_t idx = (t.row0 + t.wave + kWaves * j) * m + lcol;
        x.g = load_grad_raw<BF16, ALIGNED, CAME_NT3>(real ? g : static_cast<const void*>(&tm), real ? idx : int64_t(0), real ? lncol : kLaneCols);
        x.mo = load_mom_raw<MB16, ALIGNED>(M, idx, lncol);
        x.th = load_f32_raw<ALIGNED>(theta, idx, lncol);
        return x;
    };
    // element-wise loads (unaligned rows) need far more address registers per row in flight:
    // one row per batch there
    constexpr int U = ALIGNED ? kRows3 : 1;
    const WaveRows wr = wave_rows<U>(t);
    Row A[U], B[U];
    if (wr.nfull > 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) A[u] = load_row(u);
    }

    // 1^T R_t from the per-workgroup sums finalize 2 left (every wave, same order, same bits)
    float sqrt_sum_R = 1.f;
    if (came)
        sqrt_sum_R = static_cast<float>(sqrt(wave_sum_list(
            reinterpret_cast<const double*>(scratch + tm.off_fpart) + tm.f_row_wgs, tm.f_row_wgs)));
    const float row_scale_u = sc->sqrt_sum_r * sc->kappa;
    const float row_scale_s = came ? sqrt_sum_R * h.lr : h.lr;

    // per-row factors kappa rsqrt(r_i / 1^T r) and eta rsqrt(R_i / 1^T R) of the tile's rows,
    // once, into LDS (inside the row loop: LDS broadcast reads, no global load to wait for)
    for (int i = threadIdx.x; i < mrows; i += kWorkgroup) {
        rowfac[i] = rsqrtf(r[mrow0 + i]) * row_scale_u;
        rowfac[TR + i] = came ? rsqrtf(R[mrow0 + i]) * row_scale_s : row_scale_s;
    }

    float b[8], Bc[8];
    {
        float cv[8];
        if constexpr (SPLIT) unpack(load_f32_pair(c, sg.ca, sg.cb), cv);
        else unpack(load_f32_raw<ALIGNED>(c, lcol, lncol), cv);
#pragma unroll
        for (int e = 0; e < 8; ++e) b[e] = (SPLIT || e < t.ncol) ? rsqrtf(cv[e]) : 0.f;
        if (came) {
            if constexpr (SPLIT) unpack(load_f32_pair(C, sg.ca, sg.cb), cv);
            else unpack(load_f32_raw<ALIGNED>(C, lcol, lncol), cv);
#pragma unroll
            for (int e = 0; e < 8; ++e) Bc[e] = (SPLIT || e < t.ncol) ? rsqrtf(cv[e]) : 0.f;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) Bc[e] = 1.f;
        }
    }
    __syncthreads();

    auto consume_row = [&](const Row& row, int j) {
        if constexpr (SPLIT) {
            const SplitStep st = split_step<FOLDED>(t, sg, j, pitch, mrows, m);
            // the factors of the two groups' rows (a missing row's lanes compute on a copy and store nothing)
            const int ra = st.oka ? st.rowa : st.rowa - 1, rb = st.okb ? st.rowb : st.rowb - 1;
            const float aa = rowfac[ra], ab = rowfac[rb];
            const float Aa = rowfac[TR + ra], Ab = rowfac[TR + rb];
            float x[8], mo[8], th[8], mn[8], tn[8];
            unpack<BF16>(row.g, x);
            unpack<MB16>(row.mo, mo);
            unpack(row.th, th);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float uh = (x[e] * (e < 4 ? aa : ab)) * b[e];
                mn[e] = fmaf(h.beta1, mo[e], h.one_minus_beta1 * uh);
                tn[e] = fmaf(th[e], h.decay, -((mn[e] * (e < 4 ? Aa : Ab)) * Bc[e]));
            }
            // (where the stores go: the same places the loads came from, unless the row is missing)
            const int64_t base = (t.row0 + t.wave + kWaves * j) * pitch;
            const int64_t ia = base + sg.va, ib = base + sg.vb;
            if constexpr (MB16) store_bf16_pair(M, ia, ib, st.oka, st.okb, mn);
            else store_f32_pair(M, ia, ib, st.oka, st.okb, mn);
            store_f32_pair(theta, ia, ib, st.oka, st.okb, tn);
            if constexpr (COPY16) store_bf16_pair(theta16, ia, ib, st.oka, st.okb, tn);
            return;
        }
        const int i = t.wave + kWaves * j;
        const float a = rowfac[i];
        const float Ar = rowfac[TR + i];
        float x[8], mo[8], th[8], mn[8], tn[8];
        unpack<BF16>(row.g, x);
        unpack<MB16>(row.mo, mo);
        unpack(row.th, th);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float uh = (x[e] * a) * b[e];
            mn[e] = fmaf(h.beta1, mo[e], h.one_minus_beta1 * uh);
            tn[e] = fmaf(th[e], h.decay, -((mn[e] * Ar) * Bc[e]));
        }
        const int64_t idx = (t.row0 + i) * m + t.col;
        if constexpr (ALIGNED && FULL) {
            store_mom<MB16, true>(M, idx, kLaneCols, mn);
            store_f32x8<true>(theta, idx, kLaneCols, tn);
            if constexpr (COPY16) store_bf16x8<true>(theta16, idx, kLaneCols, tn);
        } else {
            store_mom<MB16, ALIGNED>(M, idx, t.ncol, mn);
            store_f32x8<ALIGNED>(theta, idx, t.ncol, tn);
            if constexpr (COPY16) store_bf16x8<ALIGNED>(theta16, idx, t.ncol, tn);
        }
    };

    if (wr.nfull > 0) {
        for (int k = 0;; k += 2) {
            const int kb = min(k + 1, wr.nfull - 1);
#pragma unroll
            for (int u = 0; u < U; ++u) B[u] = load_row(kb * U + u, k + 1 < wr.nfull);
#pragma unroll
            for (int u = 0; u < U; ++u) consume_row(A[u], k * U + u);
            if (k + 1 >= wr.nfull) break;
            const int ka = min(k + 2, wr.nfull - 1);
#pragma unroll
            for (int u = 0; u < U; ++u) A[u] = load_row(ka * U + u, k + 2 < wr.nfull);
#pragma unroll
            for (int u = 0; u < U; ++u) consume_row(B[u], (k + 1) * U + u);
            if (k + 2 >= wr.nfull) break;
        }
    }
    for (int j = wr.nfull * U; j < wr.cnt; ++j) consume_row(load_row(j), j);
}

#ifndef CAME_WAVES3
#define CAME_WAVES3 3
#endif
// The first vec_count workgroups of a sweep-3 launch update whole 1-D parameters instead (work
// items vec_begin...): that work is independent of the matrices and latency-bound, so at the
// front of the step's longest launch it is over long before the tiles are, instead of costing a
// launch of its own.
#define CAME_SWEEP3_KERNEL(NAME, BF16, ALIGNED, MB16, WAVES)                                              \
    __global__ __launch_bounds__(kWorkgroup) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES)))     \
    void NAME(DeviceTables tb, int32_t item_begin, int32_t vec_begin, int32_t vec_count,            \
              int32_t reverse, SweepHyper h, FinalizeHyper fh)                                      \
    {                                                                                               \
        extern __shared__ __attribute__((aligned(16))) float rowfac_f32[];                          \
        if (static_cast<int32_t>(blockIdx.x) < vec_count) {                                         \
            vector_item(tb, vec_begin + blockIdx.x, h, fh, reinterpret_cast<double*>(rowfac_f32));  \
            return;                                                                                 \
        }                                                                                           \
        const int32_t ntile = static_cast<int32_t>(gridDim.x) - vec_count;                          \
        const int32_t ord = xcd_item(static_cast<int32_t>(blockIdx.x) - vec_count, ntile);          \
        const WorkItem it = tb.items[item_begin + (reverse ? ntile - 1 - ord : ord)];               \
        const TensorMeta& tm = tb.metas[it.tensor];                                                 \
        const bool folded = ALIGNED && it.kind == 5;                                                \
        const TileGeom t = folded ? folded_geom(tm, it, tm.tile_rows3) : tile_geom(tm, it, tm.tile_rows3); \
        const bool full = static_cast<int64_t>(it.cb + 1) * kTileCols <= tm.m;                      \
        float* theta = static_cast<float*>(tb.theta[it.tensor]);                         \
        void* theta16 = tb.theta16[it.tensor];                       \
        const void* g = tb.grad[it.tensor];                    \
        const TensorScalars* sc = tb.scalars + it.tensor;                                           \
        if (folded) {                                                                               \
            if (theta16) sweep3_tile<BF16, ALIGNED, ALIGNED ? kTileFolded : kTileFull, true, MB16>(tm, it, t, g, theta, theta16, tb.state, tb.scratch, sc, h, rowfac_f32); \
            else sweep3_tile<BF16, ALIGNED, ALIGNED ? kTileFolded : kTileFull, false, MB16>(tm, it, t, g, theta, theta16, tb.state, tb.scratch, sc, h, rowfac_f32); \
        } else if (!ALIGNED || full) {                                                              \
            if (theta16) sweep3_tile<BF16, ALIGNED, kTileFull, true, MB16>(tm, it, t, g, theta, theta16, tb.state, tb.scratch, sc, h, rowfac_f32); \
            else sweep3_tile<BF16, ALIGNED, kTileFull, false, MB16>(tm, it, t, g, theta, theta16, tb.state, tb.scratch, sc, h, rowfac_f32); \
        } else {                                                                                    \
            if (theta16) sweep3_tile<BF16, ALIGNED, kTileRagged, true, MB16>(tm, it, t, g, theta, theta16, tb.state, tb.scratch, sc, h, rowfac_f32); \
            else sweep3_tile<BF16, ALIGNED, kTileRagged, false, MB16>(tm, it, t, g, theta, theta16, tb.state, tb.scratch, sc, h, rowfac_f32); \
        }                                                                                           \
    }
CAME_SWEEP3_KERNEL(sweep3_bf16_kernel, true, true, false, CAME_WAVES3)
CAME_SWEEP3_KERNEL(sweep3_f32_kernel, false, true, false, 3)
CAME_SWEEP3_KERNEL(sweep3_bf16_unaligned_kernel, true, false, false, 4)
CAME_SWEEP3_KERNEL(sweep3_f32_unaligned_kernel, false, false, false, 4)
#ifndef CAME_WAVES3M
#define CAME_WAVES3M CAME_WAVES3
#endif
CAME_SWEEP3_KERNEL(sweep3_bf16_mbf16_kernel, true, true, true, CAME_WAVES3M)
CAME_SWEEP3_KERNEL(sweep3_f32_mbf16_kernel, false, true, true, 3)
CAME_SWEEP3_KERNEL(sweep3_bf16_mbf16_unaligned_kernel, true, false, true, 4)
CAME_SWEEP3_KERNEL(sweep3_f32_mbf16_unaligned_kernel, false, false, true, 4)

// ---------------------------------------------------------------- placement probe

// The memory traffic of sweep 2 or sweep 3 without their arithmetic, in the sweeps' tile
// order, contents unchanged.  Used to find out how well the caller's placement of theta, g
// and of the state blob suits the memory system before any state exists (see
// came_probe_placement).
//   mode 0: read every theta and M entry of the matrix tiles (and g when with_g) and write the
//           same theta and M bits back: sweep 3's streams;
//   mode 1: read g and M, write nothing: sweep 2's streams.
// Loaded gradient bits are folded into a word that is stored only if it equals a value it
// cannot take, so that the loads stay.
__global__ __launch_bounds__(kWorkgroup) void placement_probe_kernel(DeviceTables tb, int32_t item_begin,
                                                                     int32_t mode, int32_t with_g)
{
    const WorkItem it = tb.items[item_begin + xcd_item(blockIdx.x, gridDim.x)];
    const TensorMeta& tm = tb.metas[it.tensor];
    if (!(tm.flags & kFlagAligned)) return;
    const bool folded = it.kind == 5 || it.kind == 6;
    const int32_t tile_rows = it.kind == 4 || it.kind == 5 ? tm.tile_rows3 : tm.tile_rows;
    const TileGeom t = folded ? folded_geom(tm, it, tile_rows) : tile_geom(tm, it, tile_rows);
    // the lane's two groups of 4 columns, as the sweeps take them: split ownership unless the
    // matrix ends inside the tile (then 8 consecutive columns, or none)
    const bool ragged = !folded && static_cast<int64_t>(it.cb + 1) * kTileCols > tm.m;
    if (ragged && t.ncol == 0) return;
    const SplitGeom sg = folded ? split_geom<true>(tm, it, t) : split_geom<false>(tm, it, t);
    const int64_t pitch = folded ? 2 * tm.m : tm.m;
    const int mrows = folded ? static_cast<int>(min(static_cast<int64_t>(2 * t.nrows), tm.n - 2 * t.row0)) : t.nrows;
    float* theta = static_cast<float*>(tb.theta[it.tensor]);
    float* M = tb.state + tm.off_M;
    const bool mb16 = tm.flags & kFlagBf16Momentum, gb16 = tm.flags & kFlagBf16Grad;
    const CAME_GLOBAL uint16_t* g16 = glob(static_cast<const uint16_t*>(tb.grad[it.tensor]));
    CAME_GLOBAL uint16_t* m16 = glob(reinterpret_cast<uint16_t*>(M));
    uint32_t sink = 0u;
    for (int j = 0; t.wave + kWaves * j < t.nrows; ++j) {
        int64_t ia, ib;
        bool oka = true, okb = true;
        if (ragged) {
            ia = (t.row0 + t.wave + kWaves * j) * pitch + t.col;
            ib = ia + 4;
        } else {
            const SplitStep st = folded ? split_step<true>(t, sg, j, pitch, mrows, tm.m) : split_step<false>(t, sg, j, pitch, mrows, tm.m);
            ia = st.ia; ib = st.ib; oka = st.oka; okb = st.okb;  // (a missing row's lanes read the row before it and store nothing)
        }
        if (with_g) {
            if (gb16) {
                const u32x2 a = __builtin_nontemporal_load((const CAME_GLOBAL u32x2*)(g16 + ia));
                const u32x2 b = __builtin_nontemporal_load((const CAME_GLOBAL u32x2*)(g16 + ib));
                sink ^= a.x ^ a.y ^ b.x ^ b.y;
            } else {
                const u32x4 a = __builtin_nontemporal_load((const CAME_GLOBAL u32x4*)(g16 + 2 * ia));
                const u32x4 b = __builtin_nontemporal_load((const CAME_GLOBAL u32x4*)(g16 + 2 * ib));
                sink ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w;
            }
        }
        u32x4 m0 = {0u, 0u, 0u, 0u}, m1 = m0;
        if (mb16) {
            const u32x2 a = *(const CAME_GLOBAL u32x2*)(m16 + ia), b = *(const CAME_GLOBAL u32x2*)(m16 + ib);
            m0.x = a.x; m0.y = a.y; m1.x = b.x; m1.y = b.y;
        } else {
            m0 = *(const CAME_GLOBAL u32x4*)(m16 + 2 * ia);
            m1 = *(const CAME_GLOBAL u32x4*)(m16 + 2 * ib);
        }
        if (mode == 0) {
            f32x4 t0 = *(const CAME_GLOBAL f32x4*)(glob(theta) + ia), t1 = *(const CAME_GLOBAL f32x4*)(glob(theta) + ib);
            // opaque to the optimiser, so that the stores of just-loaded values are kept
            asm volatile("" : "+v"(m0), "+v"(m1), "+v"(t0), "+v"(t1));
            if (oka) {
                if (mb16) *(CAME_GLOBAL u32x2*)(m16 + ia) = u32x2{m0.x, m0.y};
                else *(CAME_GLOBAL u32x4*)(m16 + 2 * ia) = m0;
                *(CAME_GLOBAL f32x4*)(glob(theta) + ia) = t0;
            }
            if (okb) {
                if (mb16) *(CAME_GLOBAL u32x2*)(m16 + ib) = u32x2{m1.x, m1.y};
                else *(CAME_GLOBAL u32x4*)(m16 + 2 * ib) = m1;
                *(CAME_GLOBAL f32x4*)(glob(theta) + ib) = t1;
            }
        } else {
            sink ^= m0.x ^ m0.y ^ m0.z ^ m0.w ^ m1.x ^ m1.y ^ m1.z ^ m1.w;
        }
    }
    // never true: the per-workgroup scalars hold four floats and four zero words per tensor
    if (sink == 0x7fc12345u && tb.scalars[it.tensor].pad_[0] == 0xffffffffu) tb.scalars[it.tensor].pad_[1] = sink;
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
    if (blocks > kNumCus * 32) blocks = kNumCus * 32;
    if (blocks == 0) blocks = 1;
    fill_zero_kernel<<<dim3(static_cast<unsigned>(blocks)), dim3(kWorkgroup), 0, s>>>(
        reinterpret_cast<f32x4*>(p), n4, p + n4 * 4, ntail);
    return hipGetLastError();
}

hipError_t launch_fill_zero_bytes(void* p, size_t bytes, hipStream_t s)
{
    return launch_fill_zero(static_cast<float*>(p), bytes / sizeof(float), s);
}

hipError_t launch_placement_probe(const DeviceTables& t, int32_t item_begin, int32_t item_end, int mode,
                                  bool with_g, hipStream_t s)
{
    if (item_end <= item_begin) return hipSuccess;
    placement_probe_kernel<<<dim3(item_end - item_begin), dim3(kWorkgroup), 0, s>>>(t, item_begin, mode, with_g ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_vectors(const DeviceTables& t, int32_t item_begin, int32_t item_end,
                          const SweepHyper& h, const FinalizeHyper& fh, hipStream_t s)
{
    if (item_end <= item_begin) return hipSuccess;
    vector_kernel<<<dim3(item_end - item_begin), dim3(kWorkgroup), 0, s>>>(t, item_begin, h, fh);
    return hipGetLastError();
}

hipError_t launch_long_vectors(const DeviceTables& t, int32_t item_begin, int32_t item_end,
                               const SweepHyper& h, const FinalizeHyper& fh, hipStream_t s)
{
    if (item_end <= item_begin) return hipSuccess;
    const dim3 grid(item_end - item_begin), block(kWorkgroup);
    long_vector_kernel<<<grid, block, 0, s>>>(t, item_begin, 1, h, fh);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    long_vector_kernel<<<grid, block, 0, s>>>(t, item_begin, 2, h, fh);
    return hipGetLastError();
}

hipError_t launch_sweep1(const DeviceTables& t, int variant, int32_t lds_rows, int32_t item_begin,
                         int32_t item_end, hipStream_t s)
{
    if (item_end <= item_begin) return hipSuccess;
    const dim3 grid(item_end - item_begin), block(kWorkgroup);
    const size_t dyn = sizeof(float) * static_cast<size_t>(lds_rows);  // row sums of one tile
    switch (variant & 3) {  // sweep 1 does not touch M
        case 0: sweep1_bf16_kernel<<<grid, block, dyn, s>>>(t, item_begin); break;
        case 1: sweep1_f32_kernel<<<grid, block, dyn, s>>>(t, item_begin); break;
        case 2: sweep1_bf16_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin); break;
        default: sweep1_f32_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin); break;
    }
    return hipGetLastError();
}

hipError_t launch_finalize1(const DeviceTables& t, int32_t fin_begin, int32_t fin_end,
                            const FinalizeHyper& h, hipStream_t s)
{
    if (fin_end <= fin_begin) return hipSuccess;
    finalize1_kernel<<<dim3(fin_end - fin_begin), dim3(kWorkgroup), 0, s>>>(t, fin_begin, h);
    return hipGetLastError();
}

hipError_t launch_sweep2(const DeviceTables& t, int variant, int32_t algo, int32_t lds_rows,
                         int32_t item_begin, int32_t item_end, bool reverse, bool stream_m, hipStream_t s)
{
    if (item_end <= item_begin) return hipSuccess;
    const dim3 grid(item_end - item_begin), block(kWorkgroup);
    // three row statistics (double) and one row factor (float) per row of the matrix in a tile
    const size_t dyn = (sizeof(double) * 3 + sizeof(float)) * static_cast<size_t>(lds_rows);
    const int32_t rev = reverse ? 1 : 0;
    if (algo == CAME_ALGO_CAME && stream_m && !(variant & 2)) {
        switch (variant) {
            case 0: sweep2_bf16_ntm_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 1: sweep2_f32_ntm_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 4: sweep2_bf16_mbf16_ntm_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            default: sweep2_f32_mbf16_ntm_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
        }
    } else if (algo == CAME_ALGO_CAME) {
        switch (variant) {
            case 0: sweep2_bf16_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 1: sweep2_f32_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 2: sweep2_bf16_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 3: sweep2_f32_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 4: sweep2_bf16_mbf16_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 5: sweep2_f32_mbf16_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 6: sweep2_bf16_mbf16_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            default: sweep2_f32_mbf16_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
        }
    } else {
        switch (variant & 3) {
            case 0: sweep2_adafactor_bf16_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 1: sweep2_adafactor_f32_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            case 2: sweep2_adafactor_bf16_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
            default: sweep2_adafactor_f32_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, rev, lds_rows); break;
        }
    }
    return hipGetLastError();
}

hipError_t launch_finalize2(const DeviceTables& t, int32_t fin_begin, int32_t fin_end,
                            const FinalizeHyper& h, hipStream_t s)
{
    if (fin_end <= fin_begin) return hipSuccess;
    finalize2_kernel<<<dim3(fin_end - fin_begin), dim3(kWorkgroup), 0, s>>>(t, fin_begin, h);
    return hipGetLastError();
}

hipError_t launch_sweep3(const DeviceTables& t, int variant, int32_t tile_rows, int32_t item_begin,
                         int32_t item_end, int32_t vec_begin, int32_t vec_end, bool reverse, const SweepHyper& h,
                         const FinalizeHyper& fh, hipStream_t s)
{
    if (item_end <= item_begin) return hipSuccess;
    const int32_t vec_count = vec_end - vec_begin;
    const int32_t rev = reverse ? 1 : 0;
    const dim3 grid(item_end - item_begin + vec_count), block(kWorkgroup);
    // two factors per row of the matrix in a tile (a folded tile holds two of them per row of
    // its own); a whole-vector item needs 4 doubles
    const size_t dyn = std::max(sizeof(float) * 4 * static_cast<size_t>(tile_rows), sizeof(double) * 4);
    switch (variant) {
        case 0: sweep3_bf16_kernel<<<grid, block, dyn, s>>>(t, item_begin, vec_begin, vec_count, rev, h, fh); break;
        case 1: sweep3_f32_kernel<<<grid, block, dyn, s>>>(t, item_begin, vec_begin, vec_count, rev, h, fh); break;
        case 2: sweep3_bf16_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, vec_begin, vec_count, rev, h, fh); break;
        case 3: sweep3_f32_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, vec_begin, vec_count, rev, h, fh); break;
        case 4: sweep3_bf16_mbf16_kernel<<<grid, block, dyn, s>>>(t, item_begin, vec_begin, vec_count, rev, h, fh); break;
        case 5: sweep3_f32_mbf16_kernel<<<grid, block, dyn, s>>>(t, item_begin, vec_begin, vec_count, rev, h, fh); break;
        case 6: sweep3_bf16_mbf16_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, vec_begin, vec_count, rev, h, fh); break;
        default: sweep3_f32_mbf16_unaligned_kernel<<<grid, block, dyn, s>>>(t, item_begin, vec_begin, vec_count, rev, h, fh); break;
    }
    return hipGetLastError();
}

}  // namespace came
