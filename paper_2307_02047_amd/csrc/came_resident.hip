// On-chip path of the CAME step (Algorithm 2) for matrices whose tiles all fit on the chip at once.
//
// Algorithm 2 has two points at which a whole-tensor quantity must be complete before any element
// can go on: r_t and c_t (row and column sums of g^2 + eps1) before any u_t = g / sqrt(v_t), and
// RMS(u_t) of Eq. 1 before any u^_t, M_t, theta_t.  The streaming kernels therefore read g three
// times and M twice.  Here a matrix is cut into tiles of 16 rows x 512 columns, one per workgroup,
// all of them on the chip at the same time; each workgroup keeps its tile of g and of M_{t-1} in
// LDS while the workgroups of the matrix exchange their partial sums through memory and wait for
// each other.  g, M and theta then cross the memory bus once per step (read g, M, theta; write M,
// theta).
//
// Per tile (lane l owns columns 8l..8l+7, wave w rows w, w+4, w+8, w+12):
//   phase 1   load g and M_{t-1}; partial row sums (tile's 512 columns) and column sums (tile's 16 rows) of g^2
//   meeting 1
//   reduce 1  the workgroups of column block 0 add the row partials of their 16 rows -> r_t and
//             the row block's share of 1^T r_t; the workgroups of a column block share out its 512
//             columns and add the column partials over the row blocks -> c_t
//   meeting 2
//   phase 2   u = g / sqrt(v_t); partial row/column sums of u^2, u M, M^2 (binary64),
//             tile sum of u^2
//   meeting 3
//   reduce 2  kappa of Eq. 1 from the tile sums (every workgroup, same order, same bits); R_t and
//             C_t like r_t and c_t, from  sum U = beta1^2 (kappa^2 sum u^2 - 2 kappa sum u M + sum M^2)
//   meeting 4
//   phase 3   load theta; M_t = beta1 M_{t-1} + (1-beta1) kappa u;  theta_t = theta_{t-1} - eta M_t / sqrt(S_t)
//
// Workgroup b of the launch takes the tiles b, b + grid, b + 2 grid, ... of a list in which the
// tiles of a matrix are consecutive and no matrix has more tiles than the grid has workgroups.
// Every workgroup thus meets the matrices in list order and each at most once.  The grid is no
// larger than what the chip holds at once (the host checks it against the occupancy the runtime
// reports), so on a GPU that this launch has to itself all workgroups are resident, and among the
// matrices somebody still works on, the first in the list has all its workgroups either working on
// it or on their way to it without anything to wait for in between: no cycle of waits can form.
// Should other work hold compute units back, the missing workgroups start when that work ends, and
// the waiting ones go on then.  Each wait is bounded in time all the same: when the bound runs out
// the workgroup raises a flag, every workgroup stops waiting from then on and runs through its
// remaining tiles (all addresses are independent of loaded data), the launch ends normally and the
// host reports CAME_ETIMEOUT.
//
// What one workgroup writes and another reads inside the launch (partial sums, r, c, R, C, the
// row-block sums, the counters) goes through agent-scope atomic loads and stores: write-through
// and cache-bypassing accesses that are coherent across the chip's eight L2 caches without any
// cache-wide write-back or invalidate.  A workgroup reports in at a meeting only after all its
// waves have seen those stores acknowledged.  g, M and theta of a tile are touched by its own
// workgroup only and use ordinary accesses.  No atomics on data: results are bit-reproducible.
#include <hip/hip_runtime.h>

#include "came_device.hpp"
#include "came_kernels.h"

namespace came {
namespace {

// Relaxed atomic accesses at agent scope to device memory (global address space: the blobs are
// the caller's device allocations): coherent across the chip without a fence.
template <class T>
__device__ __forceinline__ T ld_agent(const T* p)
{
    return __hip_atomic_load(glob(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <class T>
__device__ __forceinline__ void st_agent(T* p, T v)
{
    __hip_atomic_store(glob(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ int32_t add_agent(int32_t* p, int32_t v)
{
    return __hip_atomic_fetch_add(glob(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A value that is the same in every lane, moved into scalar registers word by word.  Inside the
// persistent loop the compiler has to load the tile's descriptors with vector loads (memory has
// been written since the kernel began), and everything computed from them -- sizes, offsets,
// pointers -- would then occupy vector registers in every lane.
template <class T>
__device__ __forceinline__ T uniform(const T& x)
{
    static_assert(sizeof(T) % 4 == 0, "whole words");
    union { T v; int32_t w[sizeof(T) / 4]; } in, out;
    in.v = x;
#pragma unroll
    for (size_t k = 0; k < sizeof(T) / 4; ++k) out.w[k] = __builtin_amdgcn_readfirstlane(in.w[k]);
    return out.v;
}

// A coherent load is an ordered access: the compiler neither moves it across another one nor out
// of a conditional, and waits for it where its value is first used.  A loop "s += ld_agent(..)"
// therefore pays one full memory round trip per term.  The sums below take four terms per trip:
// four requests in straight-line code (terms beyond the end re-request the first of the four and
// are dropped), then the additions, in index order -- a fixed order, so every caller that adds
// the same list gets the same bits.
//   at(k) -> const T* is the address of term k; terms begin, begin + step, ... below end.
template <class At>
__device__ __forceinline__ double sum_agent(int begin, int end, int step, At at)
{
    double s = 0.0;
    for (int k = begin; k < end; k += 4 * step) {
        const int k1 = k + step, k2 = k + 2 * step, k3 = k + 3 * step;
        const auto v0 = ld_agent(at(k));
        const auto v1 = ld_agent(at(k1 < end ? k1 : k));
        const auto v2 = ld_agent(at(k2 < end ? k2 : k));
        const auto v3 = ld_agent(at(k3 < end ? k3 : k));
        s += static_cast<double>(v0);
        s += k1 < end ? static_cast<double>(v1) : 0.0;
        s += k2 < end ? static_cast<double>(v2) : 0.0;
        s += k3 < end ? static_cast<double>(v3) : 0.0;
    }
    return s;
}

// The same for three statistics kept `gap` elements apart (u^2, u M, M^2 of one row or column).
template <class At>
__device__ __forceinline__ void sum3_agent(int begin, int end, int step, int gap, At at, double& sP, double& sQ, double& sW)
{
    sP = sQ = sW = 0.0;
    for (int k = begin; k < end; k += 2 * step) {
        const int k1 = k + step;
        const double* p0 = at(k);
        const double* p1 = at(k1 < end ? k1 : k);
        const double a0 = ld_agent(p0), a1 = ld_agent(p0 + gap), a2 = ld_agent(p0 + 2 * gap);
        const double b0 = ld_agent(p1), b1 = ld_agent(p1 + gap), b2 = ld_agent(p1 + 2 * gap);
        sP += a0; sQ += a1; sW += a2;
        if (k1 < end) { sP += b0; sQ += b1; sW += b2; }
    }
}

// Sum of list[0..count) by one wave in a fixed order, read coherently; same bits in every wave
// that evaluates it.  Every lane of the wave must be active.
__device__ __forceinline__ double wave_sum_list_agent(const double* list, int count)
{
    const double s = sum_agent(threadIdx.x & 63, count, 64, [&](int k) { return list + k; });
    return wave_sum(s);
}

// Meeting point of the `k` workgroups of one matrix.  `met` counts the meetings of this matrix so
// far (uniform over the workgroup).  Returns with `failed` set when this or any other workgroup
// of the launch has given up a wait; from then on nobody waits any more.
__device__ __forceinline__ void meet(ResidentSync* sync, int32_t k, int32_t& met, bool& failed,
                                     const ResidentCtl& ctl, int32_t* lds_flag)
{
    // all stores of this wave acknowledged, then all waves of the workgroup here
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    met += 1;
    if (threadIdx.x == 0) {
        bool f = failed;
        const int32_t before = add_agent(&sync->arrived, 1);
        if (before + 1 == met * k) {
            st_agent(&sync->released, met);  // the last one in: everybody may go on
        } else if (!f) {
            const uint64_t t0 = wall_clock64();
            uint32_t spins = 0;
            while (ld_agent(&sync->released) < met) {
                __builtin_amdgcn_s_sleep(4);
                if ((++spins & 15u) == 0u) {
                    if (ld_agent(ctl.fail_dev) != 0) { f = true; break; }
                    if (wall_clock64() - t0 > ctl.limit_ticks) {
                        st_agent(ctl.fail_dev, 1);
                        __hip_atomic_store(ctl.fail_host, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                        f = true;
                        break;
                    }
                }
            }
        }
        *lds_flag = f ? 1 : 0;
    }
    __syncthreads();
    failed = *lds_flag != 0;
}

// The columns [j0, j1) of column block `cb` (local indices 0..511) that the workgroup of row block
// `rb` adds up after a meeting: the RB workgroups of a column block share its 512 columns out evenly.
struct ColumnShare { int j0, j1; };
__device__ __forceinline__ ColumnShare column_share(int rb, int RB)
{
    const int chunk = (kTileCols + RB - 1) / RB;
    ColumnShare s;
    s.j0 = min(rb * chunk, kTileCols);
    s.j1 = min(s.j0 + chunk, kTileCols);
    return s;
}

// How a workgroup adds up its share of columns: groups of `gsz` consecutive lanes (a power of two,
// at most a wave) take one column each, lane l of a group the row blocks l, l + gsz, ...; the
// group's lanes then add their sums in a butterfly (fixed order).  All columns of a pass -- and with
// shares of up to 16 columns that is all of them -- are thus requested at once instead of one
// column and one round trip after the other.
struct ColumnGroups { int gsz, cols_per_pass; };
__device__ __forceinline__ ColumnGroups column_groups(int share_cols)
{
    const int per = min(share_cols, static_cast<int>(kWorkgroup));
    int gsz = 64;
    while (gsz > 1 && gsz * per > kWorkgroup) gsz >>= 1;
    ColumnGroups g;
    g.gsz = gsz;
    g.cols_per_pass = kWorkgroup / gsz;
    return g;
}

// Sum over the `gsz` lanes of a group (gsz a power of two <= 64), the same value in all of them.
__device__ __forceinline__ double group_sum(double v, int gsz)
{
    for (int mask = gsz >> 1; mask >= 1; mask >>= 1) v += __shfl_xor(v, mask);
    return v;
}

constexpr int RPW = kResidentRowsPerWave;
constexpr int kHalfCols = kTileCols / 2;  // the column sums of a tile cross the waves 256 columns at a time

// The caller's buffers of the tile's matrix and the two blobs.
struct ResidentArgs {
    const void* g;
    float* theta;
    void* theta16;
    TensorScalars* sc;
    float* state;
    char* scratch;
};

// Address of a lane's 8 entries of a row: a row start that is the same for the whole wave (kept in
// scalar registers) plus a 32-bit lane offset in elements.  The accesses then take the
// scalar-base + vector-offset form and no 64-bit per-lane address is kept alive per row and array.
template <class T>
__device__ __forceinline__ CAME_GLOBAL T* lane_ptr(T* row_start, uint32_t lane_elems)
{
    return (CAME_GLOBAL T*)((CAME_GLOBAL char*)glob(row_start) + static_cast<uint64_t>(lane_elems * static_cast<uint32_t>(sizeof(T))));
}

// B16: 2-byte entries (bfloat16), else binary32.  nt: streaming load (data read once and never written).
template <bool B16>
__device__ __forceinline__ GradRaw<B16> load_row_raw(const void* row_start, uint32_t lane_elems, bool nt)
{
    GradRaw<B16> r;
    if constexpr (B16) {
        const CAME_GLOBAL u32x4* p = (const CAME_GLOBAL u32x4*)lane_ptr(static_cast<const uint16_t*>(row_start), lane_elems);
        r.v = nt ? __builtin_nontemporal_load(p) : *p;
    } else {
        const CAME_GLOBAL f32x4* p = (const CAME_GLOBAL f32x4*)lane_ptr(static_cast<const float*>(row_start), lane_elems);
        if (nt) { r.a = __builtin_nontemporal_load(p); r.b = __builtin_nontemporal_load(p + 1); }
        else { r.a = p[0]; r.b = p[1]; }
    }
    return r;
}

template <bool B16>
__device__ __forceinline__ void store_row(void* row_start, uint32_t lane_elems, const float (&x)[8])
{
    if constexpr (B16) {
        u32x4 v;
        v.x = bf16_bits(x[0]) | (bf16_bits(x[1]) << 16);
        v.y = bf16_bits(x[2]) | (bf16_bits(x[3]) << 16);
        v.z = bf16_bits(x[4]) | (bf16_bits(x[5]) << 16);
        v.w = bf16_bits(x[6]) | (bf16_bits(x[7]) << 16);
        *(CAME_GLOBAL u32x4*)lane_ptr(static_cast<uint16_t*>(row_start), lane_elems) = v;
    } else {
        CAME_GLOBAL f32x4* p = (CAME_GLOBAL f32x4*)lane_ptr(static_cast<float*>(row_start), lane_elems);
        p[0] = f32x4{x[0], x[1], x[2], x[3]};
        p[1] = f32x4{x[4], x[5], x[6], x[7]};
    }
}

// A lane's 8 entries of one row of a tile kept in LDS, as they sit in memory (row-major, 512
// entries per row; each wave reads and writes its own rows only).  B16: 2-byte entries.
template <bool B16>
__device__ __forceinline__ void lds_put(char* tile, int row, int lane, const GradRaw<B16>& r)
{
    if constexpr (B16) {
        *reinterpret_cast<u32x4*>(tile + (static_cast<size_t>(row) * kTileCols + lane * kLaneCols) * 2) = r.v;
    } else {
        f32x4* p = reinterpret_cast<f32x4*>(tile + (static_cast<size_t>(row) * kTileCols + lane * kLaneCols) * 4);
        p[0] = r.a;
        p[1] = r.b;
    }
}

template <bool B16>
__device__ __forceinline__ GradRaw<B16> lds_get(const char* tile, int row, int lane)
{
    GradRaw<B16> r;
    if constexpr (B16) {
        r.v = *reinterpret_cast<const u32x4*>(tile + (static_cast<size_t>(row) * kTileCols + lane * kLaneCols) * 2);
    } else {
        const f32x4* p = reinterpret_cast<const f32x4*>(tile + (static_cast<size_t>(row) * kTileCols + lane * kLaneCols) * 4);
        r.a = p[0];
        r.b = p[1];
    }
    return r;
}

// Column sums of a tile across its 4 waves, 256 columns at a time through `buf` ([4][256]): every
// lane hands in its 8 per-column sums `acc`, thread j of the workgroup then holds the total of
// column half*256 + j of the tile and passes it to `emit(half, j, total)`.
template <class T, class Emit>
__device__ __forceinline__ void combine_columns(T* buf, const T (&acc)[8], int wave, int lane, Emit emit)
{
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        if ((lane >> 5) == half) {
#pragma unroll
            for (int e = 0; e < 8; ++e) buf[wave * kHalfCols + (lane & 31) * kLaneCols + e] = acc[e];
        }
        __syncthreads();
        {
            const int j = threadIdx.x;  // kWorkgroup == kHalfCols
            emit(half, j, (buf[j] + buf[kHalfCols + j]) + (buf[2 * kHalfCols + j] + buf[3 * kHalfCols + j]));
        }
        __syncthreads();
    }
}
static_assert(kWorkgroup == kHalfCols, "one thread per column of a half tile");

template <bool BF16, bool MB16>
__device__ __forceinline__ void resident_tile(const ResidentArgs& ra, const TensorMeta& tm, const WorkItem& it,
                                              const SweepHyper& h, const FinalizeHyper& fh, const ResidentCtl& ctl,
                                              char* ldsG /* [16][512] gradient entries */,
                                              char* ldsM /* [16][512] momentum entries */, double* lds /* [4][256] */,
                                              double* lds4, double* rowbuf /* [3][16] */, float* rowfac /* [2][16] */,
                                              float* colfac /* [512] */,
                                              int32_t* lds_flag, bool& failed, int32_t k /* tile's place in the launch's list */)
{
    const TileGeom t = tile_geom(tm, it);
    const int64_t n = tm.n, m = tm.m;
    const int RB = tm.RB, CB = tm.CB;
    const void* g = ra.g;
    float* theta = ra.theta;
    void* theta16 = ra.theta16;
    char* scratch = ra.scratch;
    float* r = ra.state + tm.off_r;
    float* c = ra.state + tm.off_c;
    float* R = ra.state + tm.off_R;
    float* C = ra.state + tm.off_C;
    float* M = ra.state + tm.off_M;
    TensorScalars* sc = ra.sc;
    ResidentSync* sync = reinterpret_cast<ResidentSync*>(scratch + tm.off_sync);
    double* fpart = reinterpret_cast<double*>(scratch + tm.off_fpart);  // [0,RB): sums of r; [RB,2RB): of R
    // Partial sums travel through one region per workgroup of the grid: tile k of the list is held
    // by workgroup k mod grid, and a workgroup moves on to its next tile only after the last meeting
    // of the current tile's matrix, when nobody reads that matrix's partial sums any more.
    const int32_t first_k = k - (it.rb * CB + it.cb);  // the matrix's tile (0, 0)
    auto region_of = [&](int rb, int cb) -> char* {
        return ctl.regions + static_cast<size_t>((first_k + rb * CB + cb) % static_cast<int32_t>(gridDim.x)) * kResidentRegionBytes;
    };
    char* mine_region = region_of(it.rb, it.cb);
    const bool lane_valid = t.ncol > 0;
    const int64_t col0 = static_cast<int64_t>(it.cb) * kTileCols;
    // lanes beyond the last column load from the tile's first columns (which exist) and are masked
    const uint32_t lane_elems = lane_valid ? static_cast<uint32_t>(t.lane * kLaneCols) : 0u;
    const bool first_tile = it.rb == 0 && it.cb == 0;
    const ColumnShare share = column_share(it.rb, RB);
    int32_t met = 0;

    // the wave's u-th row within the tile; start of the part of that row that lies in this tile,
    // as an element offset into the matrix (the same for the whole wave; rows beyond the tile's
    // last load from that last row and are masked)
    auto row_of = [&](int u) { return t.wave + kWaves * u; };
    auto row_start = [&](int u) {
        const int i = min(row_of(u), t.nrows - 1);
        return (t.row0 + i) * m + col0;
    };
    auto live = [&](int u) { return lane_valid && row_of(u) < t.nrows; };

    // ---------------------------------------------------------------- phase 1
    {
        GradRaw<BF16> G[RPW];
        GradRaw<MB16> Mo[RPW];
#pragma unroll
        for (int u = 0; u < RPW; ++u)
            G[u] = load_row_raw<BF16>(static_cast<const char*>(g) + row_start(u) * (BF16 ? 2 : 4), lane_elems, true);
        // M_{t-1} of the tile does not depend on anything the others produce: requested right away
#pragma unroll
        for (int u = 0; u < RPW; ++u)
            Mo[u] = load_row_raw<MB16>(reinterpret_cast<const char*>(M) + row_start(u) * (MB16 ? 2 : 4), lane_elems, false);
        float* rowsum = reinterpret_cast<float*>(rowbuf);
        float cacc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) cacc[e] = 0.f;
#pragma unroll
        for (int u = 0; u < RPW; ++u) {
            lds_put<BF16>(ldsG, row_of(u), t.lane, G[u]);  // stays there until phase 3
            float x[8];
            unpack<BF16>(G[u], x);
            const bool ok = live(u);
            float racc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x[e] = ok ? x[e] : 0.f;
                racc = fmaf(x[e], x[e], racc);
                cacc[e] = fmaf(x[e], x[e], cacc[e]);
            }
            racc = wave_sum_lane63(racc);
            if (t.lane == 63) rowsum[row_of(u)] = racc;
        }
        float* rowpart = reinterpret_cast<float*>(mine_region + kResidentRowpartOffset);
        float* colpart = reinterpret_cast<float*>(mine_region + kResidentColpartOffset);
        combine_columns(reinterpret_cast<float*>(lds), cacc, t.wave, t.lane, [&](int half, int j, float total) {
            const int jj = half * kHalfCols + j;
            if (col0 + jj < m) st_agent(&colpart[jj], total);
        });
        if (static_cast<int>(threadIdx.x) < t.nrows) st_agent(&rowpart[threadIdx.x], rowsum[threadIdx.x]);
#pragma unroll
        for (int u = 0; u < RPW; ++u) lds_put<MB16>(ldsM, row_of(u), t.lane, Mo[u]);  // until phase 3
    }
    meet(sync, tm.ntiles, met, failed, ctl, lds_flag);

    // ---------------------------------------------------------------- reduce 1: r_t, c_t
    const ColumnGroups cg = column_groups(share.j1 - share.j0);
    const bool has_columns = share.j0 < share.j1 && col0 + share.j0 < m;
    const bool row_thread = it.cb == 0 && static_cast<int>(threadIdx.x) < t.nrows;
    {
        // the first four row partials are requested before the columns' and used after them, so
        // that the workgroups that do both pay one round trip for both
        float rv[4] = {0.f, 0.f, 0.f, 0.f};
        float r_old = 0.f;
        if (row_thread) {
            r_old = glob(r)[t.row0 + threadIdx.x];  // last step's: an ordinary load
#pragma unroll
            for (int q = 0; q < 4; ++q)
                rv[q] = ld_agent(reinterpret_cast<const float*>(region_of(it.rb, min(q, CB - 1)) + kResidentRowpartOffset) + threadIdx.x);
        }
        if (has_columns) {
            for (int base = share.j0; base < share.j1; base += cg.cols_per_pass) {
                const int j = base + static_cast<int>(threadIdx.x) / cg.gsz, li = static_cast<int>(threadIdx.x) % cg.gsz;
                const bool ok = j < share.j1 && col0 + j < m;
                const int jc = ok ? j : share.j0;
                const float c_old = glob(c)[col0 + jc];
                double s = sum_agent(li, RB, cg.gsz, [&](int rb) {
                    return reinterpret_cast<const float*>(region_of(rb, it.cb) + kResidentColpartOffset) + jc;
                });
                s = group_sum(s, cg.gsz);
                if (ok && li == 0) {
                    s += static_cast<double>(n) * fh.eps1;
                    st_agent(&c[col0 + j], static_cast<float>(fh.beta2 * static_cast<double>(c_old) + fh.one_minus_beta2 * s));
                }
            }
        }
        if (it.cb == 0 && t.wave == 0) {  // (a tile has 16 rows: they all sit in the first wave)
            double mine = 0.0;
            if (row_thread) {
                double s = 0.0;
#pragma unroll
                for (int q = 0; q < 4; ++q) s += q < CB ? static_cast<double>(rv[q]) : 0.0;
                s += sum_agent(4, CB, 1, [&](int cb) {
                    return reinterpret_cast<const float*>(region_of(it.rb, cb) + kResidentRowpartOffset) + threadIdx.x;
                });
                s += static_cast<double>(m) * fh.eps1;
                const float rn = static_cast<float>(fh.beta2 * static_cast<double>(r_old) + fh.one_minus_beta2 * s);
                st_agent(&r[t.row0 + threadIdx.x], rn);
                mine = static_cast<double>(rn);
            }
            const double total = wave_sum(mine);
            if (t.lane == 0) st_agent(&fpart[it.rb], total);
        }
    }
    meet(sync, tm.ntiles, met, failed, ctl, lds_flag);

    // ---------------------------------------------------------------- phase 2: statistics of u
    float* rs_r = rowfac;                      // rsqrt(r_i) of the tile's rows (0 beyond the last)
    float* row_S = rowfac + kResidentRows;     // eta rsqrt(R_i / 1^T R) (phase 3)
    float b[8];  // rsqrt(c_j) of this lane's columns
    float sqrt_sum_r;
    {
        // the tile's column factors, two columns per thread, and row factors, all requested in one
        // go (columns and rows beyond the matrix re-request its last ones and are zeroed)
        const int64_t ca = min(col0 + threadIdx.x, m - 1), cb2 = min(col0 + kHalfCols + threadIdx.x, m - 1);
        const float c_a = ld_agent(&c[ca]), c_b = ld_agent(&c[cb2]);
        const float r_i = ld_agent(&r[min(t.row0 + (threadIdx.x & (kResidentRows - 1)), n - 1)]);
        sqrt_sum_r = static_cast<float>(sqrt(wave_sum_list_agent(fpart, RB)));
        colfac[threadIdx.x] = col0 + threadIdx.x < m ? rsqrtf(c_a) : 0.f;
        colfac[kHalfCols + threadIdx.x] = col0 + kHalfCols + threadIdx.x < m ? rsqrtf(c_b) : 0.f;
        if (threadIdx.x < kResidentRows) rs_r[threadIdx.x] = static_cast<int>(threadIdx.x) < t.nrows ? rsqrtf(r_i) : 0.f;
        if (first_tile && threadIdx.x == 0) sc->sqrt_sum_r = sqrt_sum_r;
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) b[e] = colfac[t.lane * kLaneCols + e];
    }
    {
        double cP[8], cQ[8], cW[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) cP[e] = cQ[e] = cW[e] = 0.0;
#pragma unroll 1
        for (int u = 0; u < RPW; ++u) {
            const int i = row_of(u);
            const float a = rs_r[i] * sqrt_sum_r;  // rsqrt(r_i / 1^T r); 0 for rows beyond the tile's last
            const bool ok = live(u);
            float x[8], mo[8];
            unpack<BF16>(lds_get<BF16>(ldsG, i, t.lane), x);
            unpack<MB16>(lds_get<MB16>(ldsM, i, t.lane), mo);
            double rP = 0.0, rQ = 0.0, rW = 0.0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float uf = ok ? (x[e] * a) * b[e] : 0.f;  // u_ij = g_ij / sqrt(v_ij)
                const double du = static_cast<double>(uf);
                const double dm = static_cast<double>(ok ? mo[e] : 0.f);
                rP = fma(du, du, rP); rQ = fma(du, dm, rQ); rW = fma(dm, dm, rW);
                cP[e] = fma(du, du, cP[e]); cQ[e] = fma(du, dm, cQ[e]); cW[e] = fma(dm, dm, cW[e]);
            }
            rP = wave_sum_lane63(rP); rQ = wave_sum_lane63(rQ); rW = wave_sum_lane63(rW);
            if (t.lane == 63) { rowbuf[i] = rP; rowbuf[kResidentRows + i] = rQ; rowbuf[2 * kResidentRows + i] = rW; }
        }
        double* rowpart = reinterpret_cast<double*>(mine_region + kResidentRowpartOffset);  // [3][16]
        double* colpart = reinterpret_cast<double*>(mine_region + kResidentColpartOffset);  // [3][512]
        auto emit = [&](int q) {
            return [&, q](int half, int j, double total) {
                const int jj = half * kHalfCols + j;
                if (col0 + jj < m) st_agent(&colpart[q * kTileCols + jj], total);
            };
        };
        combine_columns(lds, cP, t.wave, t.lane, emit(0));
        combine_columns(lds, cQ, t.wave, t.lane, emit(1));
        combine_columns(lds, cW, t.wave, t.lane, emit(2));
        double p = 0.0;
        if (static_cast<int>(threadIdx.x) < t.nrows) {
            const int i = threadIdx.x;
            p = rowbuf[i];
            st_agent(&rowpart[i], p);
            st_agent(&rowpart[kResidentRows + i], rowbuf[kResidentRows + i]);
            st_agent(&rowpart[2 * kResidentRows + i], rowbuf[2 * kResidentRows + i]);
        }
        p = block_sum(p, lds4);
        if (threadIdx.x == 0) st_agent(reinterpret_cast<double*>(mine_region + kResidentTilePOffset), p);
    }
    // theta_{t-1} of the tile, requested before the third meeting: it arrives while the workgroup waits
    GradRaw<false> Th[RPW];
#pragma unroll
    for (int u = 0; u < RPW; ++u) Th[u] = load_row_raw<false>(theta + row_start(u), lane_elems, false);
    meet(sync, tm.ntiles, met, failed, ctl, lds_flag);

    // ---------------------------------------------------------------- reduce 2: kappa, R_t, C_t
    float kappa_f;
    {
        // requested in one go: the tiles' sums of u^2, the first two column blocks' row partials,
        // (inside the column pass) the column partials; kappa is needed only where they are combined
        const double pp = sum_agent(threadIdx.x, tm.ntiles, kWorkgroup, [&](int q) {
            return reinterpret_cast<const double*>(
                ctl.regions + static_cast<size_t>((first_k + q) % static_cast<int32_t>(gridDim.x)) * kResidentRegionBytes + kResidentTilePOffset);
        });
        double rP[2] = {0.0, 0.0}, rQ[2] = {0.0, 0.0}, rW[2] = {0.0, 0.0};
        float R_old = 0.f;
        if (row_thread) {
            R_old = glob(R)[t.row0 + threadIdx.x];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const double* rp = reinterpret_cast<const double*>(region_of(it.rb, min(q, CB - 1)) + kResidentRowpartOffset) + threadIdx.x;
                rP[q] = ld_agent(rp); rQ[q] = ld_agent(rp + kResidentRows); rW[q] = ld_agent(rp + 2 * kResidentRows);
            }
        }
        const double P = block_sum(pp, lds4);
        const double rms = sqrt(P / (static_cast<double>(n) * static_cast<double>(m)));
        const double kappa = 1.0 / fmax(1.0, rms / fh.clip_d);
        kappa_f = static_cast<float>(kappa);
        if (first_tile && threadIdx.x == 0) {
            sc->kappa = kappa_f;
            sc->rms_u = static_cast<float>(rms);
        }
        const double b1sq = fh.beta1 * fh.beta1, k2 = kappa * kappa, km2 = -2.0 * kappa;
        if (has_columns) {
            for (int base = share.j0; base < share.j1; base += cg.cols_per_pass) {
                const int j = base + static_cast<int>(threadIdx.x) / cg.gsz, li = static_cast<int>(threadIdx.x) % cg.gsz;
                const bool ok = j < share.j1 && col0 + j < m;
                const int jc = ok ? j : share.j0;
                const float C_old = glob(C)[col0 + jc];
                double sP, sQ, sW;
                sum3_agent(li, RB, cg.gsz, kTileCols, [&](int rb) {
                    return reinterpret_cast<const double*>(region_of(rb, it.cb) + kResidentColpartOffset) + jc;
                }, sP, sQ, sW);
                sP = group_sum(sP, cg.gsz); sQ = group_sum(sQ, cg.gsz); sW = group_sum(sW, cg.gsz);
                if (ok && li == 0) {
                    double U = b1sq * ((k2 * sP + km2 * sQ) + sW);
                    U = U < 0.0 ? 0.0 : U;  // rounding of the three-term sum; a NaN stays a NaN
                    U += static_cast<double>(n) * fh.eps2;
                    st_agent(&C[col0 + j], static_cast<float>(fh.beta3 * static_cast<double>(C_old) + fh.one_minus_beta3 * U));
                }
            }
        }
        if (it.cb == 0 && t.wave == 0) {
            double mine = 0.0;
            if (row_thread) {
                double sP, sQ, sW;
                sum3_agent(2, CB, 1, kResidentRows, [&](int cb) {
                    return reinterpret_cast<const double*>(region_of(it.rb, cb) + kResidentRowpartOffset) + threadIdx.x;
                }, sP, sQ, sW);
                sP = (rP[0] + (CB > 1 ? rP[1] : 0.0)) + sP;
                sQ = (rQ[0] + (CB > 1 ? rQ[1] : 0.0)) + sQ;
                sW = (rW[0] + (CB > 1 ? rW[1] : 0.0)) + sW;
                double U = b1sq * ((k2 * sP + km2 * sQ) + sW);
                U = U < 0.0 ? 0.0 : U;
                U += static_cast<double>(m) * fh.eps2;
                const float Rn = static_cast<float>(fh.beta3 * static_cast<double>(R_old) + fh.one_minus_beta3 * U);
                st_agent(&R[t.row0 + threadIdx.x], Rn);
                mine = static_cast<double>(Rn);
            }
            const double total = wave_sum(mine);
            if (t.lane == 0) st_agent(&fpart[RB + it.rb], total);
        }
    }
    meet(sync, tm.ntiles, met, failed, ctl, lds_flag);

    // ---------------------------------------------------------------- phase 3: M_t, theta_t
    {
        const int64_t ca = min(col0 + threadIdx.x, m - 1), cb2 = min(col0 + kHalfCols + threadIdx.x, m - 1);
        const float C_a = ld_agent(&C[ca]), C_b = ld_agent(&C[cb2]);
        const float R_i = ld_agent(&R[min(t.row0 + (threadIdx.x & (kResidentRows - 1)), n - 1)]);
        const float sqrt_sum_R = static_cast<float>(sqrt(wave_sum_list_agent(fpart + RB, RB)));
        if (first_tile && threadIdx.x == 0) sc->sqrt_sum_R = sqrt_sum_R;
        const float row_scale_u = sqrt_sum_r * kappa_f;
        const float row_scale_s = sqrt_sum_R * h.lr;
        colfac[threadIdx.x] = col0 + threadIdx.x < m ? rsqrtf(C_a) : 0.f;
        colfac[kHalfCols + threadIdx.x] = col0 + kHalfCols + threadIdx.x < m ? rsqrtf(C_b) : 0.f;
        if (threadIdx.x < kResidentRows) row_S[threadIdx.x] = static_cast<int>(threadIdx.x) < t.nrows ? rsqrtf(R_i) * row_scale_s : 0.f;
        __syncthreads();
        float Bc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) Bc[e] = colfac[t.lane * kLaneCols + e];
#pragma unroll
        for (int u = 0; u < RPW; ++u) {
            const int i = row_of(u);
            const float a = rs_r[i] * row_scale_u;  // kappa rsqrt(r_i / 1^T r)
            const float Ar = row_S[i];
            float x[8], mo[8], th[8], mn[8], tn[8];
            unpack<BF16>(lds_get<BF16>(ldsG, i, t.lane), x);
            unpack<MB16>(lds_get<MB16>(ldsM, i, t.lane), mo);
            unpack<false>(Th[u], th);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float uh = (x[e] * a) * b[e];
                mn[e] = fmaf(h.beta1, mo[e], h.one_minus_beta1 * uh);
                tn[e] = fmaf(th[e], h.decay, -((mn[e] * Ar) * Bc[e]));
            }
            if (live(u)) {  // (then row_start(u) is the row itself and lane_elems this lane's own columns)
                store_row<MB16>(reinterpret_cast<char*>(M) + row_start(u) * (MB16 ? 2 : 4), lane_elems, mn);
                store_row<false>(theta + row_start(u), lane_elems, tn);
                if (theta16) store_row<true>(static_cast<char*>(theta16) + row_start(u) * 2, lane_elems, tn);
            }
        }
    }

    // through with this matrix; the last workgroup to leave clears the counters for the next launch
    if (threadIdx.x == 0) {
        const int32_t before = add_agent(&sync->departed, 1);
        if (before == tm.ntiles - 1) {
            st_agent(&sync->arrived, 0);
            st_agent(&sync->released, 0);
            st_agent(&sync->departed, 0);
        }
    }
}

// Kept out of line: its registers are then the callee's own and do not compete with the tiles'.
// Arguments by value: a reference would force the kernel's own copies of them into memory.
__device__ __attribute__((noinline)) void resident_vector_item(DeviceTables tb, int32_t item, SweepHyper h,
                                                               FinalizeHyper fh, double* lds4)
{
    vector_item(tb, item, h, fh, lds4);
}

// The tables arrive as separate read-only, non-aliased kernel arguments (not inside DeviceTables):
// only then does the compiler know that the stores and atomics of one tile cannot change what the
// next tile's descriptors say, and keeps descriptors, offsets and pointers in scalar registers.
#define CAME_RESIDENT_KERNEL(NAME, BF16, MB16)                                                              \
    __global__ __launch_bounds__(kWorkgroup)                                                                \
    __attribute__((amdgpu_waves_per_eu(kResidentWgsPerCu, kResidentWgsPerCu)))                              \
    void NAME(const TensorMeta* __restrict__ metas, const WorkItem* __restrict__ items,                     \
              void* const* __restrict__ theta_tab, const void* const* __restrict__ grad_tab,                \
              void* const* __restrict__ theta16_tab, TensorScalars* scalars, float* state, char* scratch,   \
              int32_t item_begin, int32_t item_count, int32_t vec_begin, int32_t vec_count,                 \
              SweepHyper h, FinalizeHyper fh, ResidentCtl ctl)                                              \
    {                                                                                                       \
        __shared__ __attribute__((aligned(16))) char ldsG[kResidentRows * kTileCols * (BF16 ? 2 : 4)];      \
        __shared__ __attribute__((aligned(16))) char ldsM[kResidentRows * kTileCols * (MB16 ? 2 : 4)];      \
        __shared__ double lds[kWaves * kHalfCols];                                                          \
        __shared__ double lds4[4];                                                                          \
        __shared__ double rowbuf[3 * kResidentRows];                                                        \
        __shared__ float rowfac[2 * kResidentRows];                                                         \
        __shared__ __attribute__((aligned(16))) float colfac[kTileCols];                                    \
        __shared__ int32_t lds_flag;                                                                        \
        bool failed = false;                                                                                \
        for (int32_t k = blockIdx.x; k < item_count; k += gridDim.x) {                                      \
            const WorkItem it = uniform(items[item_begin + k]);                                             \
            const TensorMeta tm = uniform(metas[it.tensor]);                                                \
            ResidentArgs a;                                                                                 \
            a.g = grad_tab[it.tensor];                                                                      \
            a.theta = static_cast<float*>(theta_tab[it.tensor]);                                            \
            a.theta16 = theta16_tab[it.tensor];                                                             \
            a.sc = scalars + it.tensor;                                                                     \
            a.state = state;                                                                                \
            a.scratch = scratch;                                                                            \
            resident_tile<BF16, MB16>(uniform(a), tm, it, h, fh, ctl, ldsG, ldsM, lds, lds4, rowbuf, rowfac, colfac, \
                                      &lds_flag, failed, k);                                                \
            __syncthreads();                                                                                \
        }                                                                                                   \
        /* whole 1-D parameters riding along: dealt out from the last workgroup downwards, away from */     \
        /* the workgroups that hold one more tile than the others                                     */     \
        for (int32_t v = static_cast<int32_t>(gridDim.x) - 1 - static_cast<int32_t>(blockIdx.x); v < vec_count; \
             v += gridDim.x) {                                                                              \
            DeviceTables tb;                                                                                \
            tb.metas = metas; tb.items = items; tb.fins = nullptr; tb.scalars = scalars;                    \
            tb.theta = theta_tab; tb.grad = grad_tab; tb.theta16 = theta16_tab;                             \
            tb.state = state; tb.scratch = scratch;                                                         \
            resident_vector_item(tb, vec_begin + v, h, fh, lds4);                                           \
        }                                                                                                   \
    }
CAME_RESIDENT_KERNEL(resident_bf16_kernel, true, false)
CAME_RESIDENT_KERNEL(resident_f32_kernel, false, false)
CAME_RESIDENT_KERNEL(resident_bf16_mbf16_kernel, true, true)
CAME_RESIDENT_KERNEL(resident_f32_mbf16_kernel, false, true)

const void* resident_entry(int variant)
{
    switch (variant) {
        case 0: return reinterpret_cast<const void*>(&resident_bf16_kernel);
        case 1: return reinterpret_cast<const void*>(&resident_f32_kernel);
        case 4: return reinterpret_cast<const void*>(&resident_bf16_mbf16_kernel);
        case 5: return reinterpret_cast<const void*>(&resident_f32_mbf16_kernel);
        default: return nullptr;
    }
}

}  // namespace

hipError_t resident_occupancy(int variant, int* workgroups_per_cu)
{
    const void* f = resident_entry(variant);
    if (!f) return hipErrorInvalidValue;
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(workgroups_per_cu, f, kWorkgroup, 0);
}

hipError_t launch_resident(const DeviceTables& t, int variant, int32_t item_begin, int32_t item_end,
                           int32_t vec_begin, int32_t vec_end, const SweepHyper& h, const FinalizeHyper& fh,
                           const ResidentCtl& ctl, hipStream_t s)
{
    if (item_end <= item_begin) return hipSuccess;
    const void* f = resident_entry(variant);
    if (!f) return hipErrorInvalidValue;
    const TensorMeta* metas = t.metas;
    const WorkItem* items = t.items;
    void* const* theta_tab = t.theta;
    const void* const* grad_tab = t.grad;
    void* const* theta16_tab = t.theta16;
    TensorScalars* scalars = t.scalars;
    float* state = t.state;
    char* scratch = t.scratch;
    int32_t ib = item_begin, ic = item_end - item_begin;
    int32_t vb = vec_begin, vc = vec_end > vec_begin ? vec_end - vec_begin : 0;
    SweepHyper sh = h;
    FinalizeHyper fhh = fh;
    ResidentCtl c = ctl;
    void* args[] = {&metas, &items, &theta_tab, &grad_tab, &theta16_tab, &scalars, &state, &scratch,
                    &ib, &ic, &vb, &vc, &sh, &fhh, &c};
    const int32_t grid = ic < kResidentGrid ? ic : kResidentGrid;
    return hipLaunchKernel(f, dim3(static_cast<unsigned>(grid)), dim3(kWorkgroup), args, 0, s);
}

}  // namespace came
