// Host-only driver for the launch planner, built with -fsanitize=address,undefined by
// tests/test_sanitizers.py.  Reads tensor descriptors ("rows cols ndim grad_dtype" per line)
// from the file named on the command line, builds the plan and re-checks on the host what the
// kernels assume about it: every work item and finalize item names a tensor and a block that
// exist, every state array and every scratch region lies inside its blob, none overlap.
//
//   plan_driver <descs.txt> <tile_rows> <algo> <group_elements> <momentum_dtype> <vector_rule> <resident> <tile_rows3>
//
// Prints "rc state_bytes scratch_bytes items fins groups" and exits 0, or exits 3 with a message
// when an invariant is broken.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "came_plan.h"

using namespace came;

namespace {

struct Range { long long lo, hi; const char* what; int tensor; };

int fail(const char* what, long long a, long long b)
{
    std::fprintf(stderr, "plan invariant broken: %s (%lld, %lld)\n", what, a, b);
    return 3;
}

int check_disjoint(std::vector<Range>& r, long long limit, const char* blob)
{
    std::sort(r.begin(), r.end(), [](const Range& a, const Range& b) { return a.lo < b.lo; });
    long long end = 0;
    for (const Range& x : r) {
        if (x.lo < end) { std::fprintf(stderr, "%s: %s of tensor %d overlaps its predecessor\n", blob, x.what, x.tensor); return 3; }
        if (x.hi > limit) { std::fprintf(stderr, "%s: %s of tensor %d leaves the blob\n", blob, x.what, x.tensor); return 3; }
        end = x.hi;
    }
    return 0;
}

}  // namespace

int main(int argc, char** argv)
{
    if (argc != 9) return 2;
    std::vector<came_tensor_desc> descs;
    if (FILE* f = std::fopen(argv[1], "r")) {
        long long rows, cols;
        int ndim, dt;
        while (std::fscanf(f, "%lld %lld %d %d", &rows, &cols, &ndim, &dt) == 4)
            descs.push_back(came_tensor_desc{rows, cols, ndim, dt});
        std::fclose(f);
    } else {
        return 2;
    }
    came_options o{};
    o.tile_rows = std::atoi(argv[2]);
    o.algo = std::atoi(argv[3]);
    o.group_elements = std::atoll(argv[4]);
    o.momentum_dtype = std::atoi(argv[5]);
    o.vector_rule = std::atoi(argv[6]);
    o.resident = std::atoi(argv[7]);
    o.tile_rows3 = std::atoi(argv[8]);
    Plan p;
    const int rc = build_plan(descs.empty() ? nullptr : descs.data(), static_cast<int32_t>(descs.size()), &o, &p);
    if (rc != CAME_OK) {
        std::printf("%d 0 0 0 0 0\n", rc);
        return 0;
    }
    const long long count = static_cast<long long>(descs.size());
    const bool mb16 = o.momentum_dtype == CAME_MOMENTUM_BF16;

    // state blob: M | r | c | R | C per tensor, in floats
    std::vector<Range> st;
    for (int t = 0; t < count; ++t) {
        const TensorMeta& tm = p.metas[t];
        const long long nm = tm.n * tm.m;
        st.push_back(Range{tm.off_M, tm.off_M + (mb16 ? (nm + 1) / 2 : nm), "M", t});
        st.push_back(Range{tm.off_r, tm.off_r + tm.n, "r", t});
        st.push_back(Range{tm.off_R, tm.off_R + tm.n, "R", t});
        if (!(tm.flags & kFlagVector)) {
            st.push_back(Range{tm.off_c, tm.off_c + tm.m, "c", t});
            st.push_back(Range{tm.off_C, tm.off_C + tm.m, "C", t});
        } else if (tm.off_c != -1 || tm.off_C != -1 || tm.m != 1) {
            return fail("vector with column statistics", t, tm.m);
        }
    }
    if (int e = check_disjoint(st, static_cast<long long>(p.state_bytes / sizeof(float)), "state")) return e;

    // scratch blob: tables, pointer slots, partial sums (bytes)
    std::vector<Range> sc;
    auto add = [&](size_t off, size_t bytes, const char* what, int t) {
        sc.push_back(Range{static_cast<long long>(off), static_cast<long long>(off + bytes), what, t});
    };
    add(p.off_metas, sizeof(TensorMeta) * count, "metas", -1);
    add(p.off_items, sizeof(WorkItem) * p.items.size(), "items", -1);
    add(p.off_fins, sizeof(FinalizeItem) * p.fins.size(), "fins", -1);
    add(p.off_scalars, sizeof(TensorScalars) * count, "scalars", -1);
    add(p.off_sync, sizeof(ResidentSync) * (count + 1), "on-chip counters", -1);
    if (p.off_sync < p.off_scalars + sizeof(TensorScalars) * count) return fail("counters not behind the scalars", p.off_sync, p.off_scalars);
    if (p.n_resident > 0) add(p.off_regions, kResidentRegionBytes * kResidentGrid, "on-chip partial-sum regions", -1);
    add(p.off_ptrs, p.ptr_slot_bytes * kPtrSlots, "pointer slots", -1);
    if (p.ptr_slot_bytes < sizeof(void*) * kPtrArrays * count) return fail("pointer slot too small", p.ptr_slot_bytes, count);
    for (int t = 0; t < count; ++t) {
        const TensorMeta& tm = p.metas[t];
        if (tm.flags & kFlagVector) {
            if (tm.ntiles > 0) {
                add(tm.off_tileP, sizeof(double) * tm.ntiles, "chunk sums", t);
                if (static_cast<long long>(tm.ntiles) * tm.tile_rows < tm.n) return fail("long vector not covered", t, tm.n);
                if (tm.ntiles > kMaxVectorChunks || tm.tile_rows % kWorkgroup) return fail("long vector chunking", tm.ntiles, tm.tile_rows);
            } else if (tm.n > kFusedVectorMax) {
                return fail("long vector without chunks", t, tm.n);
            }
            continue;
        }
        if (static_cast<long long>(tm.CB) * kTileCols < tm.m || static_cast<long long>(tm.CB - 1) * kTileCols >= tm.m)
            return fail("column blocks", tm.CB, tm.m);
        if (tm.flags & kFlagFolded) {
            // two "row blocks" (the pairs' first rows, the pairs' second rows) per row block of the ceil(n/2) x 2m view
            const long long nv = (tm.n + 1) / 2;
            if (tm.RB % 2 || static_cast<long long>(tm.RB / 2) * tm.tile_rows < nv || static_cast<long long>(tm.RB / 2 - 1) * tm.tile_rows >= nv)
                return fail("row blocks of a folded matrix", tm.RB, tm.n);
            if (tm.ntiles != tm.RB / 2 * (2 * tm.m / kTileCols)) return fail("tile count of a folded matrix", tm.ntiles, t);
        } else {
            if (static_cast<long long>(tm.RB) * tm.tile_rows < tm.n || static_cast<long long>(tm.RB - 1) * tm.tile_rows >= tm.n)
                return fail("row blocks", tm.RB, tm.n);
            if (tm.ntiles != tm.RB * tm.CB) return fail("tile count", tm.ntiles, t);
        }
        if (tm.off_sync != static_cast<long long>(p.off_sync + sizeof(ResidentSync) * t)) return fail("counter slot", t, tm.off_sync);
        if (tm.flags & kFlagResident) {
            // all tiles of the matrix on the chip at once, aligned rows, Algorithm 2, no finalize items
            if (tm.tile_rows != kResidentRows || tm.ntiles > kResidentGrid || !(tm.flags & kFlagAligned) || p.algo != CAME_ALGO_CAME)
                return fail("on-chip matrix does not qualify", t, tm.ntiles);
            if (tm.f_row_wgs != tm.RB || tm.f_col_wgs != 0) return fail("on-chip row-block sums", tm.f_row_wgs, tm.f_col_wgs);
            add(tm.off_fpart, sizeof(double) * 2 * tm.RB, "row-block sums", t);
            continue;
        }
        if (static_cast<long long>(tm.f_row_wgs) * kWorkgroup < tm.n || static_cast<long long>(tm.f_col_wgs) * kFinalizeCols < tm.m)
            return fail("finalize coverage", tm.f_row_wgs, tm.f_col_wgs);
        add(tm.off_rowpart, sizeof(double) * 3 * tm.n * tm.CB, "row partials", t);
        add(tm.off_colpart, sizeof(double) * 3 * tm.RB * tm.m, "column partials", t);
        add(tm.off_tileP, sizeof(double) * tm.ntiles, "tile sums", t);
        add(tm.off_fpart, sizeof(double) * 2 * tm.f_row_wgs, "finalize sums", t);
    }
    if (int e = check_disjoint(sc, static_cast<long long>(p.scratch_bytes), "scratch")) return e;

    // work items: each matrix tile exactly once, inside its group's variant range; vectors once
    std::vector<long long> seen(count, 0);
    std::vector<long long> seen3(count, 0);  // elements covered by the update sweep's items
    for (const Group& g : p.groups) {
        for (int v = 0; v < kVariants; ++v)
            for (int32_t k = g.var_begin[v]; k < g.var_end[v]; ++k) {
                const WorkItem& it = p.items[k];
                if (it.tensor < g.tensor_begin || it.tensor >= g.tensor_end || (it.kind != 0 && it.kind != 6)) return fail("tile item", k, it.tensor);
                const TensorMeta& tm = p.metas[it.tensor];
                if ((it.kind == 6) != ((tm.flags & kFlagFolded) != 0)) return fail("tile item kind", it.kind, tm.flags);
                if (it.kind == 6) {
                    // folded: ceil(n/2) rows of 2m columns; the finalize kernels count two row blocks per row block of that view
                    const long long RBv = ((tm.n + 1) / 2 + tm.tile_rows - 1) / tm.tile_rows, CBv = 2 * tm.m / kTileCols;
                    if (tm.RB != 2 * RBv || tm.ntiles != RBv * CBv || tm.CB != (tm.m + kTileCols - 1) / kTileCols)
                        return fail("folded matrix blocks", tm.RB, tm.ntiles);
                    if (variant_of(tm.flags) != v || it.rb < 0 || it.rb >= RBv || it.cb < 0 || it.cb >= CBv)
                        return fail("folded tile item block", it.rb, it.cb);
                    ++seen[it.tensor];
                    continue;
                }
                if (variant_of(tm.flags) != v || it.rb < 0 || it.rb >= tm.RB || it.cb < 0 || it.cb >= tm.CB)
                    return fail("tile item block", it.rb, it.cb);
                ++seen[it.tensor];
            }
        // the update sweep's own cut: every streaming matrix's rows and columns covered exactly once
        for (int v = 0; v < kVariants; ++v)
            for (int32_t k = g.var3_begin[v]; k < g.var3_end[v]; ++k) {
                const WorkItem& it = p.items[k];
                if (it.tensor < g.tensor_begin || it.tensor >= g.tensor_end || (it.kind != 4 && it.kind != 5)) return fail("update-sweep item", k, it.tensor);
                const TensorMeta& tm = p.metas[it.tensor];
                if (tm.tile_rows3 < 4 || tm.tile_rows3 % 4 != 0) return fail("update-sweep tile height", it.tensor, tm.tile_rows3);
                if ((it.kind == 5) != ((tm.flags & kFlagFolded) != 0)) return fail("update-sweep item kind", it.kind, tm.flags);
                if (it.kind == 5) {
                    // folded: the matrix as ceil(n/2) rows of 2m columns; aligned rows, the width an odd multiple of 256
                    if (!(tm.flags & kFlagAligned) || (tm.flags & (kFlagVector | kFlagResident)) || variant_of(tm.flags) != v ||
                        tm.m % kTileCols != kTileCols / 2)
                        return fail("folded matrix", it.tensor, tm.m);
                    const long long nv = (tm.n + 1) / 2, RB3 = (nv + tm.tile_rows3 - 1) / tm.tile_rows3, CB3 = 2 * tm.m / kTileCols;
                    if (it.rb < 0 || it.rb >= RB3 || it.cb < 0 || it.cb >= CB3) return fail("folded item block", it.rb, it.cb);
                    const long long v0 = static_cast<long long>(it.rb) * tm.tile_rows3, v1 = std::min<long long>(v0 + tm.tile_rows3, nv);
                    for (long long vr = v0; vr < v1; ++vr)
                        for (long long c0 = static_cast<long long>(it.cb) * kTileCols; c0 < static_cast<long long>(it.cb + 1) * kTileCols; c0 += kLaneCols) {
                            const long long row = 2 * vr + (c0 >= tm.m ? 1 : 0);
                            if (c0 < tm.m && c0 + kLaneCols > tm.m) return fail("a lane's columns straddle two rows", it.tensor, c0);
                            if (row < tm.n) seen3[it.tensor] += kLaneCols;
                        }
                    continue;
                }
                const long long RB3 = (tm.n + tm.tile_rows3 - 1) / tm.tile_rows3;
                if ((tm.flags & (kFlagVector | kFlagResident)) || variant_of(tm.flags) != v || it.rb < 0 || it.rb >= RB3 ||
                    it.cb < 0 || it.cb >= tm.CB)
                    return fail("update-sweep item block", it.rb, it.cb);
                const long long rows = std::min<long long>(tm.tile_rows3, tm.n - static_cast<long long>(it.rb) * tm.tile_rows3);
                const long long cols = std::min<long long>(kTileCols, tm.m - static_cast<long long>(it.cb) * kTileCols);
                seen3[it.tensor] += rows * cols;
            }
        for (int v = 0; v < kVariants; ++v) {
            int32_t last_tensor = -1, expect = 0;
            for (int32_t k = g.res_begin[v]; k < g.res_end[v]; ++k) {
                const WorkItem& it = p.items[k];
                if (it.tensor < g.tensor_begin || it.tensor >= g.tensor_end || it.kind != 3) return fail("on-chip item", k, it.tensor);
                const TensorMeta& tm = p.metas[it.tensor];
                if (!(tm.flags & kFlagResident) || variant_of(tm.flags) != v || (v & 2)) return fail("on-chip item variant", k, v);
                // the tiles of a matrix are consecutive, in (row block, column block) order, matrices in list order
                if (it.tensor != last_tensor) {
                    if (it.tensor < last_tensor || expect != 0) return fail("on-chip matrices out of order", k, it.tensor);
                    last_tensor = it.tensor;
                    expect = tm.ntiles;
                }
                if (it.rb * tm.CB + it.cb != tm.ntiles - expect) return fail("on-chip tile order", it.rb, it.cb);
                --expect;
                ++seen[it.tensor];
            }
            if (expect != 0) return fail("on-chip matrix cut short", v, expect);
        }
        {
            bool any = false;
            for (int v = 0; v < kVariants; ++v) any = any || g.res_end[v] > g.res_begin[v];
            const bool want = any && g.fin_end == g.fin_begin && g.vec_end > g.vec_begin;
            if (g.vectors_with_resident != want) return fail("vectors riding with the on-chip launch", g.vectors_with_resident, want);
        }
        for (int32_t k = g.vec_begin; k < g.vec_end; ++k) {
            const WorkItem& it = p.items[k];
            if (it.kind != 1 || !(p.metas[it.tensor].flags & kFlagVector) || p.metas[it.tensor].n > kFusedVectorMax)
                return fail("vector item", k, it.tensor);
            ++seen[it.tensor];
        }
        for (int32_t k = g.lvec_begin; k < g.lvec_end; ++k) {
            const WorkItem& it = p.items[k];
            if (it.kind != 2 || it.rb < 0 || it.rb >= p.metas[it.tensor].ntiles) return fail("chunk item", k, it.tensor);
            ++seen[it.tensor];
        }
        for (int32_t k = g.fin_begin; k < g.fin_end; ++k) {
            const FinalizeItem& fi = p.fins[k];
            const TensorMeta& tm = p.metas[fi.tensor];
            if (fi.tensor < g.tensor_begin || fi.tensor >= g.tensor_end) return fail("finalize item tensor", k, fi.tensor);
            if (fi.chunk < 0 || fi.chunk >= (fi.kind == 0 ? tm.f_row_wgs : tm.f_col_wgs)) return fail("finalize item chunk", k, fi.chunk);
        }
    }
    for (int t = 0; t < count; ++t) {
        const TensorMeta& tm = p.metas[t];
        const long long want = (tm.flags & kFlagVector) ? (tm.ntiles > 0 ? tm.ntiles : 1) : tm.ntiles;
        if (seen[t] != want) return fail("tensor covered a wrong number of times", seen[t], want);
        const long long want3 = (tm.flags & (kFlagVector | kFlagResident)) ? 0 : tm.n * tm.m;
        if (seen3[t] != want3) return fail("update sweep covers a wrong number of elements", seen3[t], want3);
    }
    std::printf("%d %zu %zu %zu %zu %zu\n", rc, p.state_bytes, p.scratch_bytes, p.items.size(), p.fins.size(), p.groups.size());
    return 0;
}
