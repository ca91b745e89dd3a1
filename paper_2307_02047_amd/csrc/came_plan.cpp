// Host-only planner: argument validation, state-blob layout (Algorithm 2's
// M, r, c, R, C per tensor), scratch layout and the tile tables that turn each
// phase of the step into one grouped launch over all tensors.
#include "came_plan.h"

#include <algorithm>
#include <cmath>

namespace came {

namespace {

constexpr int64_t kAlignFloats = 64;  // 256-byte alignment of every state array
// Most work items (and finalize items) a plan may have: they are indexed with 32-bit integers on
// the device and a launch takes one workgroup per item.  2^26 is twenty times what a
// 6.7-billion-parameter list needs at the smallest tile height.
constexpr int64_t kMaxItems = int64_t(1) << 26;

// Rows per tile of the update sweep when the caller does not choose.  Measured on lists from 1e8
// to 6.7e9 parameters with one row per batch: 12 rows (three per wave) are fastest or equal
// everywhere -- over 16 rows by 0.5 % where theta and M lie in different regions of the address
// space and by 1 to 2 % where they lie in the same one; at 8 rows the per-tile prologue shows
// (+3 %); with 64 and more the read-and-write stream pair slows down by up to 20 % in the same
// region.  With the momentum stored as bfloat16 (fewer bytes per row) the optimum is 16 rows
// (2 % faster than 32, 1 % faster than 12).
constexpr int32_t kDefaultTileRows3 = 12, kDefaultTileRows3Bf16Momentum = 16;
constexpr size_t kAlignBytes = 256;

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
inline size_t round_up_sz(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Rows per tile of sweeps 1 and 2 when the caller does not choose: the largest power of two up
// to 1024 that still yields six tiles per compute unit (256 CUs).  A tile of these sweeps costs
// 20 to 25 us beyond its streaming (a chain of dependent loads under load before its first row --
// work item, descriptor, r, c -- and the combination and storing of its partial sums after its
// last), so tiles should be as tall as the list allows: measured on BERT-base-, GPT-2-medium-,
// BERT-large- and Llama-7B-shaped lists, 128 / 256..512 / 512 / 1024 rows are the optima, and
// below five tiles per compute unit the launch's last round leaves too many of them idle.  Below
// 64 rows the column partials of a tall matrix (one per row block and column) outgrow what the
// finalize kernels add up cheaply, so a list too small for that keeps 64 rows as long as that
// still gives two tiles per compute unit, and goes lower only then.
int32_t auto_tile_rows(const came_tensor_desc* d, int32_t count, const std::vector<char>& resident)
{
    auto tiles_at = [&](int32_t tr) {
        int64_t tiles = 0;
        for (int32_t t = 0; t < count; ++t)
            if (d[t].ndim == 2 && !resident[t]) tiles += ceil_div(d[t].rows, tr) * ceil_div(d[t].cols, kTileCols);
        return tiles;
    };
    // (powers of two only: they divide the usual matrix heights, whereas e.g. 496 rows would cut a
    // 1024-row matrix into 496 + 496 + 32 and add a third more tiles, most of them nearly empty)
    for (int32_t tr = 1024; tr >= 64; tr /= 2)
        if (tiles_at(tr) >= kNumCus * 6) return tr;
    for (int32_t tr = 64; tr >= 16; tr -= 16)
        if (tiles_at(tr) >= kNumCus * 2) return tr;
    return 16;
}

}  // namespace

int validate_hyper(const came_hyper* h, double lr, int64_t step)
{
    if (!h) return CAME_EINVAL;
    const double betas[3] = {h->beta1, h->beta2, h->beta3};
    for (double b : betas)
        if (!(b >= 0.0 && b < 1.0)) return CAME_EINVAL;
    if (!(h->eps1 >= 0.0) || !std::isfinite(h->eps1)) return CAME_EINVAL;
    if (!(h->eps2 >= 0.0) || !std::isfinite(h->eps2)) return CAME_EINVAL;
    if (!(h->clip_d > 0.0) || !std::isfinite(h->clip_d)) return CAME_EINVAL;
    if (!(h->weight_decay >= 0.0) || !std::isfinite(h->weight_decay)) return CAME_EINVAL;
    if (!std::isfinite(lr)) return CAME_EINVAL;
    if (step < 1) return CAME_EINVAL;
    return CAME_OK;
}

int build_plan(const came_tensor_desc* descs, int32_t count, const came_options* opts, Plan* plan)
{
    if (!descs || !plan || count <= 0) return CAME_EINVAL;
    came_options o{};
    if (opts) o = *opts;
    if (o.resident != CAME_RESIDENT_AUTO && o.resident != CAME_RESIDENT_OFF && o.resident != CAME_RESIDENT_ON)
        return CAME_EINVAL;
    if (o.resident_wait_us < 0) return CAME_EINVAL;
    if (o.algo != CAME_ALGO_CAME && o.algo != CAME_ALGO_ADAFACTOR) return CAME_EINVAL;
    if (o.tile_rows != 0 && (o.tile_rows < 4 || o.tile_rows > 1024 || o.tile_rows % 4 != 0))
        return CAME_EINVAL;
    if (o.tile_rows3 != 0 && (o.tile_rows3 < 4 || o.tile_rows3 > 1024 || o.tile_rows3 % 4 != 0))
        return CAME_EINVAL;
    if (o.reserved != 0) return CAME_EINVAL;
    if (o.group_elements < 0) return CAME_EINVAL;
    if (o.momentum_dtype != CAME_MOMENTUM_F32 && o.momentum_dtype != CAME_MOMENTUM_BF16) return CAME_EINVAL;
    if (o.vector_rule != CAME_VECTOR_ALGORITHM2 && o.vector_rule != CAME_VECTOR_MOMENTUM_ONLY) return CAME_EINVAL;

    for (int32_t t = 0; t < count; ++t) {
        const came_tensor_desc& d = descs[t];
        if (d.ndim != 1 && d.ndim != 2) return CAME_EINVAL;
        if (d.rows <= 0 || d.cols <= 0) return CAME_EINVAL;
        if (d.ndim == 1 && d.cols != 1) return CAME_EINVAL;
        if (d.grad_dtype != CAME_GRAD_F32 && d.grad_dtype != CAME_GRAD_BF16) return CAME_EINVAL;
        if (d.rows > (int64_t(1) << 40) || d.cols > (int64_t(1) << 40)) return CAME_EINVAL;
        if (d.ndim == 1 && d.rows > (int64_t(1) << 38)) return CAME_EINVAL;  // chunk size must fit int32
        if (d.rows > (int64_t(1) << 46) / d.cols) return CAME_EINVAL;  // rows*cols <= 2^46, without forming an overflowing product
    }

    Plan& p = *plan;
    p = Plan{};
    p.descs.assign(descs, descs + count);
    p.algo = o.algo;
    p.momentum_dtype = o.momentum_dtype;
    p.resident_wait_us = o.resident_wait_us;
    // Which matrices take the on-chip path: Algorithm 2 only, rows 16-byte aligned, and all tiles of
    // the matrix on the chip at once (one per workgroup of the co-resident grid).
    std::vector<char> resident(count, 0);
    // Off unless asked for: measured on MI355X the on-chip path moves a third fewer bytes but is
    // bound by the latency of the meetings between workgroups on different dies, and ends up slower
    // than the three streaming sweeps on every list tried.
    const bool on_chip = o.resident == CAME_RESIDENT_ON;
    if (on_chip && o.algo == CAME_ALGO_CAME) {
        for (int32_t t = 0; t < count; ++t) {
            const came_tensor_desc& d = descs[t];
            if (d.ndim != 2 || d.cols % kLaneCols != 0) continue;
            const int64_t RB = ceil_div(d.rows, kResidentRows), CB = ceil_div(d.cols, kTileCols);
            if (RB <= kResidentGrid && CB <= kResidentGrid && RB * CB <= kResidentGrid) resident[t] = 1;
        }
    }
    p.tile_rows = o.tile_rows ? o.tile_rows : auto_tile_rows(descs, count, resident);
    p.tile_rows3 = o.tile_rows3 ? o.tile_rows3
                                : (o.momentum_dtype == CAME_MOMENTUM_BF16 ? kDefaultTileRows3Bf16Momentum : kDefaultTileRows3);
    {
        // counted in 64 bits before anything 32-bit is derived from them
        int64_t items = 0, fins = 0;
        for (int32_t t = 0; t < count; ++t) {
            const came_tensor_desc& d = descs[t];
            if (d.ndim == 2) {
                const int64_t RB = ceil_div(d.rows, resident[t] ? kResidentRows : p.tile_rows), CB = ceil_div(d.cols, kTileCols);
                if (RB > kMaxItems || CB > kMaxItems || RB * CB > kMaxItems) return CAME_EINVAL;
                items += RB * CB;
                if (!resident[t]) {
                    // (a folded matrix has fewer tiles than this, never more)
                    const int64_t RB3 = ceil_div(d.rows, p.tile_rows3);
                    if (RB3 > kMaxItems || RB3 * CB > kMaxItems) return CAME_EINVAL;
                    items += RB3 * CB;
                }
                fins += ceil_div(d.rows, kWorkgroup) + ceil_div(d.cols, kFinalizeCols);
            } else {
                items += d.rows <= kFusedVectorMax ? 1 : kMaxVectorChunks;
            }
            if (items > kMaxItems || fins > kMaxItems) return CAME_EINVAL;
        }
    }
    p.metas.resize(count);

    // ---- state blob: per tensor M | r | c | R | C, every array 256-byte aligned
    int64_t off = 0;
    for (int32_t t = 0; t < count; ++t) {
        const came_tensor_desc& d = descs[t];
        TensorMeta& tm = p.metas[t];
        tm = TensorMeta{};
        tm.n = d.rows;
        tm.m = d.ndim == 2 ? d.cols : 1;
        tm.flags = (d.grad_dtype == CAME_GRAD_BF16 ? kFlagBf16Grad : 0) |
                   (o.momentum_dtype == CAME_MOMENTUM_BF16 ? kFlagBf16Momentum : 0);
        const int64_t nm = tm.n * tm.m;
        p.total_elements += nm;
        // a bfloat16 M occupies half as many floats of the blob
        const int64_t m_floats = o.momentum_dtype == CAME_MOMENTUM_BF16 ? (nm + 1) / 2 : nm;
        tm.off_M = off; off = round_up(off + m_floats, kAlignFloats);
        tm.off_r = off; off = round_up(off + tm.n, kAlignFloats);
        if (d.ndim == 2) {
            tm.off_c = off; off = round_up(off + tm.m, kAlignFloats);
        } else {
            tm.off_c = -1;
        }
        tm.off_R = off; off = round_up(off + tm.n, kAlignFloats);
        if (d.ndim == 2) {
            tm.off_C = off; off = round_up(off + tm.m, kAlignFloats);
            ++p.n_matrices;
            if (tm.m % kLaneCols == 0) tm.flags |= kFlagAligned;
            if (!resident[t] && tm.m % kTileCols == kTileCols / 2) tm.flags |= kFlagFolded;
            if (resident[t]) {
                tm.flags |= kFlagResident;
                ++p.n_resident;
                p.resident_elements += nm;
            }
        } else {
            tm.off_C = -1;
            tm.flags |= kFlagVector;
            if (o.vector_rule == CAME_VECTOR_MOMENTUM_ONLY) tm.flags |= kFlagMomentumOnly;
            ++p.n_vectors;
        }
    }
    p.state_bytes = static_cast<size_t>(off) * sizeof(float);
    p.reverse_sweep2 = true;
    p.keep_tail_cached = p.total_elements <= (int64_t(1) << 29);

    // ---- groups of consecutive tensors
    {
        Group g{};
        g.tensor_begin = 0;
        int64_t acc = 0;
        for (int32_t t = 0; t < count; ++t) {
            const int64_t nm = p.metas[t].n * p.metas[t].m;
            if (o.group_elements > 0 && t > g.tensor_begin && acc + nm > o.group_elements) {
                g.tensor_end = t;
                p.groups.push_back(g);
                g = Group{};
                g.tensor_begin = t;
                acc = 0;
            }
            acc += nm;
        }
        g.tensor_end = count;
        p.groups.push_back(g);
    }

    // ---- work items and finalize items, group by group
    for (Group& g : p.groups) {
        g.fin_begin = static_cast<int32_t>(p.fins.size());
        for (int32_t t = g.tensor_begin; t < g.tensor_end; ++t) {
            TensorMeta& tm = p.metas[t];
            if (tm.flags & kFlagVector) continue;
            tm.tile_rows = (tm.flags & kFlagResident) ? kResidentRows : p.tile_rows;
            tm.tile_rows3 = p.tile_rows3;
            tm.CB = static_cast<int32_t>(ceil_div(tm.m, kTileCols));
            if (tm.flags & kFlagFolded) {
                // the view has ceil(n/2) rows of 2m columns.  The finalize kernels see every row
                // block of it as two (the pairs' first rows, the pairs' second rows) and as many
                // column blocks per row as the matrix really has.
                const int32_t RBv = static_cast<int32_t>(ceil_div(ceil_div(tm.n, 2), tm.tile_rows));
                tm.RB = 2 * RBv;
                tm.ntiles = RBv * static_cast<int32_t>(2 * tm.m / kTileCols);
                p.any_folded = true;
            } else {
                tm.RB = static_cast<int32_t>(ceil_div(tm.n, tm.tile_rows));
                tm.ntiles = tm.RB * tm.CB;
            }
            if (tm.flags & kFlagResident) {
                // no finalize launch: the workgroups of the matrix reduce their own partial sums; the
                // sums of r and of R are kept per row block
                tm.f_row_wgs = tm.RB;
                tm.f_col_wgs = 0;
                continue;
            }
            tm.f_row_wgs = static_cast<int32_t>(ceil_div(tm.n, kWorkgroup));
            tm.f_col_wgs = static_cast<int32_t>(ceil_div(tm.m, kFinalizeCols));
            for (int32_t k = 0; k < tm.f_row_wgs; ++k) p.fins.push_back(FinalizeItem{t, k, 0, 0});
            for (int32_t k = 0; k < tm.f_col_wgs; ++k) p.fins.push_back(FinalizeItem{t, k, 1, 0});
        }
        g.fin_end = static_cast<int32_t>(p.fins.size());
        for (int v = 0; v < kVariants; ++v) {
            g.var_begin[v] = static_cast<int32_t>(p.items.size());
            for (int32_t t = g.tensor_begin; t < g.tensor_end; ++t) {
                const TensorMeta& tm = p.metas[t];
                if ((tm.flags & (kFlagVector | kFlagResident)) || variant_of(tm.flags) != v) continue;
                if (tm.flags & kFlagFolded) {
                    const int32_t CBv = static_cast<int32_t>(2 * tm.m / kTileCols);
                    for (int32_t rb = 0; rb < tm.RB / 2; ++rb)
                        for (int32_t cb = 0; cb < CBv; ++cb) p.items.push_back(WorkItem{t, rb, cb, 6});
                    continue;
                }
                for (int32_t rb = 0; rb < tm.RB; ++rb)
                    for (int32_t cb = 0; cb < tm.CB; ++cb) p.items.push_back(WorkItem{t, rb, cb, 0});
            }
            g.var_end[v] = static_cast<int32_t>(p.items.size());
        }
        for (int v = 0; v < kVariants; ++v) {
            g.var3_begin[v] = static_cast<int32_t>(p.items.size());
            for (int32_t t = g.tensor_begin; t < g.tensor_end; ++t) {
                const TensorMeta& tm = p.metas[t];
                if ((tm.flags & (kFlagVector | kFlagResident)) || variant_of(tm.flags) != v) continue;
                const bool folded = tm.flags & kFlagFolded;
                const int32_t RB3 = static_cast<int32_t>(ceil_div(folded ? ceil_div(tm.n, 2) : tm.n, tm.tile_rows3));
                const int32_t CB3 = folded ? static_cast<int32_t>(2 * tm.m / kTileCols) : tm.CB;
                for (int32_t rb = 0; rb < RB3; ++rb)
                    for (int32_t cb = 0; cb < CB3; ++cb) p.items.push_back(WorkItem{t, rb, cb, folded ? 5 : 4});
            }
            g.var3_end[v] = static_cast<int32_t>(p.items.size());
        }
        g.vec_begin = static_cast<int32_t>(p.items.size());
        for (int32_t t = g.tensor_begin; t < g.tensor_end; ++t)
            if ((p.metas[t].flags & kFlagVector) && p.metas[t].n <= kFusedVectorMax)
                p.items.push_back(WorkItem{t, 0, 0, 1});
        g.vec_end = static_cast<int32_t>(p.items.size());
        g.lvec_begin = g.vec_end;
        for (int32_t t = g.tensor_begin; t < g.tensor_end; ++t) {
            TensorMeta& tm = p.metas[t];
            if (!(tm.flags & kFlagVector) || tm.n <= kFusedVectorMax) continue;
            int64_t chunk = std::max<int64_t>(kFusedVectorMax, ceil_div(tm.n, kMaxVectorChunks));
            chunk = round_up(chunk, kWorkgroup);
            tm.tile_rows = static_cast<int32_t>(chunk);
            tm.ntiles = static_cast<int32_t>(ceil_div(tm.n, chunk));
            for (int32_t k = 0; k < tm.ntiles; ++k) p.items.push_back(WorkItem{t, k, 0, 2});
        }
        g.lvec_end = static_cast<int32_t>(p.items.size());
        // on-chip path: per variant, matrix after matrix in list order, tiles of a matrix
        // consecutive.  Workgroup b of the launch takes tiles b, b + grid, ...: every workgroup
        // meets the matrices in the same order, which is what keeps the waits free of cycles.
        for (int v = 0; v < kVariants; ++v) {
            g.res_begin[v] = static_cast<int32_t>(p.items.size());
            for (int32_t t = g.tensor_begin; t < g.tensor_end; ++t) {
                const TensorMeta& tm = p.metas[t];
                if (!(tm.flags & kFlagResident) || variant_of(tm.flags) != v) continue;
                for (int32_t rb = 0; rb < tm.RB; ++rb)
                    for (int32_t cb = 0; cb < tm.CB; ++cb) p.items.push_back(WorkItem{t, rb, cb, 3});
            }
            g.res_end[v] = static_cast<int32_t>(p.items.size());
        }
        g.vectors_with_resident = g.fin_end == g.fin_begin && g.vec_end > g.vec_begin;
        if (g.vectors_with_resident) {
            bool any = false;
            for (int v = 0; v < kVariants; ++v) any = any || g.res_end[v] > g.res_begin[v];
            g.vectors_with_resident = any;
        }
    }

    // ---- scratch blob
    size_t s = 0;
    p.off_metas = s;   s = round_up_sz(s + sizeof(TensorMeta) * count, kAlignBytes);
    p.off_items = s;   s = round_up_sz(s + sizeof(WorkItem) * std::max<size_t>(p.items.size(), 1), kAlignBytes);
    p.off_fins = s;    s = round_up_sz(s + sizeof(FinalizeItem) * std::max<size_t>(p.fins.size(), 1), kAlignBytes);
    p.off_scalars = s; s = round_up_sz(s + sizeof(TensorScalars) * count, kAlignBytes);
    p.off_sync = s;    s = round_up_sz(s + sizeof(ResidentSync) * (static_cast<size_t>(count) + 1), kAlignBytes);
    p.ptr_slot_bytes = round_up_sz(sizeof(void*) * kPtrArrays * count, kAlignBytes);
    p.off_ptrs = s;    s += p.ptr_slot_bytes * kPtrSlots;
    p.off_regions = s;
    if (p.n_resident > 0) s += kResidentRegionBytes * kResidentGrid;
    p.off_partials = s;
    for (int32_t t = 0; t < count; ++t) {
        TensorMeta& tm = p.metas[t];
        if (tm.flags & kFlagVector) {
            if (tm.ntiles > 0) {  // long vector: one double per chunk
                tm.off_tileP = static_cast<int64_t>(s);
                s = round_up_sz(s + sizeof(double) * tm.ntiles, kAlignBytes);
            }
            continue;
        }
        tm.off_sync = static_cast<int64_t>(p.off_sync + sizeof(ResidentSync) * static_cast<size_t>(t));
        if (tm.flags & kFlagResident) {
            // the tiles' partial sums live in the per-workgroup regions; per matrix only the row
            // blocks' sums of r and of R
            tm.off_rowpart = tm.off_colpart = tm.off_tileP = -1;
            tm.off_fpart = static_cast<int64_t>(s);
            s = round_up_sz(s + sizeof(double) * 2 * tm.f_row_wgs, kAlignBytes);
            continue;
        }
        // sized for sweep 2 (three doubles per entry); sweep 1 reuses the front of each region
        tm.off_rowpart = static_cast<int64_t>(s);
        s = round_up_sz(s + sizeof(double) * 3 * static_cast<size_t>(tm.n) * tm.CB, kAlignBytes);
        tm.off_colpart = static_cast<int64_t>(s);
        s = round_up_sz(s + sizeof(double) * 3 * static_cast<size_t>(tm.RB) * tm.m, kAlignBytes);
        tm.off_tileP = static_cast<int64_t>(s);
        s = round_up_sz(s + sizeof(double) * tm.ntiles, kAlignBytes);
        tm.off_fpart = static_cast<int64_t>(s);
        s = round_up_sz(s + sizeof(double) * 2 * tm.f_row_wgs, kAlignBytes);
    }
    p.scratch_bytes = s;
    return CAME_OK;
}

}  // namespace came
