// Launch plan of the CAME step: plain structs shared by the host planner and
// the gfx950 kernels.  Host-only logic (validation, state layout, tile table)
// lives in came_plan.cpp and needs no GPU.
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "came.h"

namespace came {

// Geometry of a sweep tile.  A workgroup of 4 wave64s sweeps `tile_rows` rows
// of a 512-column stripe: each lane owns 8 consecutive columns (one 16-byte
// bf16 load or two 16-byte f32 loads), each wave takes every 4th row.
// The one machine this library is written for, MI355X (gfx950): 8 accelerator dies (XCDs), each
// with its own L2, to which the dispatcher deals consecutive workgroups round-robin; 32 compute
// units per die.  Everything that is tuned to the chip's shape refers to these two numbers.
constexpr int kNumXcds = 8;
constexpr int kNumCus = 256;

constexpr int kWorkgroup = 256;
constexpr int kWaves = 4;
constexpr int kLaneCols = 8;
constexpr int kTileCols = 64 * kLaneCols;  // 512

// The on-chip path (came_options.resident): one launch of kResidentGrid workgroups that are all
// on the chip at once (kResidentWgsPerCu per compute unit: what the 160 KB of LDS of a compute unit
// hold; came_init_state checks it against the occupancy the runtime reports).  A matrix is cut into
// tiles of kResidentRows x kTileCols, one per workgroup, whose gradient and momentum stay in LDS
// from the first phase to the last; a matrix qualifies when all its tiles are on the chip together.
constexpr int kResidentWgsPerCu = 2;
constexpr int kResidentGrid = kNumCus * kResidentWgsPerCu;  // 512
constexpr int kResidentRowsPerWave = 4;
constexpr int kResidentRows = kWaves * kResidentRowsPerWave;  // 16
// Partial sums of the tile a workgroup of the on-chip launch currently holds: one region per
// workgroup of the grid, reused tile after tile.  Three binary64 statistics per column and per row
// of the tile (the first phase keeps one binary32 sum each in the same place) and the tile's sum of u^2.
constexpr size_t kResidentColpartOffset = 0;
constexpr size_t kResidentRowpartOffset = sizeof(double) * 3 * kTileCols;                          // 12288
constexpr size_t kResidentTilePOffset = kResidentRowpartOffset + sizeof(double) * 3 * kResidentRows;  // 12672
constexpr size_t kResidentRegionBytes = 12800;
static_assert(kResidentTilePOffset + sizeof(double) <= kResidentRegionBytes && kResidentRegionBytes % 256 == 0, "region layout");

enum TensorFlags : int32_t {
    kFlagBf16Grad = 1,  // gradient stored as bfloat16
    kFlagVector = 2,    // 1-D parameter: unfactored update, one workgroup
    kFlagAligned = 4,   // cols % 8 == 0: every row starts 16-byte aligned -> vector loads
    kFlagBf16Momentum = 8,  // M stored as bfloat16 (off_M still counts floats from the blob's start)
    kFlagMomentumOnly = 16, // vector updated by -eta M (no instability / confidence statistics)
    kFlagResident = 32,     // matrix on the on-chip path (tile_rows = kResidentRows, no finalize items)
    kFlagFolded = 64,       // the sweeps treat the matrix as ceil(n/2) rows of 2m columns (see WorkItem); RB then
                            // counts 2 per row block of that view and ntiles its tiles
};

// Per-tensor descriptor in device memory (scratch blob).
struct TensorMeta {
    int64_t n, m;                             // rows, columns (m = 1 for vectors)
    int64_t off_M, off_r, off_c, off_R, off_C;  // float offsets into the state blob (-1: absent)
    int64_t off_rowpart;                      // byte offset in scratch: per-(row, column block) partials
    int64_t off_colpart;                      // byte offset in scratch: per-(row block, column) partials
    int64_t off_tileP;                        // byte offset in scratch: one double per tile (sum of u^2)
    int64_t off_fpart;                        // byte offset in scratch: per row-finalize workgroup, sum of its
                                              // r values [0, f_row_wgs) and of its R values [f_row_wgs, 2 f_row_wgs)
    int32_t RB, CB;                           // number of row blocks / column blocks
    int32_t tile_rows;                        // rows per row block
    int32_t ntiles;                           // RB * CB
    int32_t f_row_wgs, f_col_wgs;             // finalize workgroups covering the rows / the columns
    int32_t flags;                            // TensorFlags
    int32_t tile_rows3;                       // rows per tile of the update sweep (its own work items)
    int64_t off_sync;                         // byte offset in scratch: this matrix's ResidentSync (on-chip path)
};
static_assert(sizeof(TensorMeta) == 128, "TensorMeta layout");

// Through these the workgroups of one matrix on the on-chip path wait for each other.  Arrivals are
// counted in one memory line; the last to arrive at a meeting publishes its number in another
// line, which is the only one the waiting workgroups poll (hundreds of pollers on the line that
// also takes the atomic additions would hold those up).  All zero between launches: the last
// workgroup to leave a matrix clears them.
struct ResidentSync {
    int32_t arrived;    // workgroups that have reached a meeting point, summed over the meeting points so far
    int32_t pad0_[31];
    int32_t released;   // number of the last meeting point that everybody has reached
    int32_t pad1_[15];
    int32_t departed;   // workgroups that are through with the matrix
    int32_t pad2_[15];
};
static_assert(sizeof(ResidentSync) == 256, "ResidentSync layout");

// One workgroup of a sweep launch.
struct WorkItem {
    int32_t tensor;
    int32_t rb, cb;  // row block, column block (matrix tiles)
    int32_t kind;    // 0 = matrix tile, 1 = whole vector, 2 = chunk `rb` of a long vector,
                     // 3 = tile of a matrix on the on-chip path,
                     // 4 = matrix tile of the update sweep (row blocks of TensorMeta.tile_rows3 rows),
                     // 5 = the same for a folded matrix: a matrix whose width is an odd multiple of 256
                     //     (768 = 512 + 256 ...) is swept as ceil(n/2) rows of 2m columns -- row 2v followed
                     //     by row 2v+1, which is how they lie in memory -- so that every tile is 512 columns
                     //     wide; rb and cb count blocks of that view (row blocks of tile_rows3 rows of it),
                     // 6 = tile of a folded matrix in sweeps 1 and 2 (row blocks of tile_rows rows of the view)
};

// Vectors up to this length are updated by one workgroup in one kernel.  Longer ones are cut
// into at most kMaxVectorChunks chunks (TensorMeta.tile_rows = elements per chunk,
// TensorMeta.ntiles = number of chunks) and updated in two passes with the per-chunk sums
// of u^2 in between (TensorMeta.off_tileP).
constexpr int64_t kFusedVectorMax = 16384;
constexpr int64_t kMaxVectorChunks = 1024;

// One workgroup of a finalize launch: 256 rows of one matrix (a thread per row, adding the
// row's partials over the column blocks), or 64 columns (a wave per quarter of the row
// blocks, a lane per column: tall matrices have hundreds of row blocks to add per column).
constexpr int kFinalizeCols = 64;
struct FinalizeItem {
    int32_t tensor;
    int32_t chunk;  // rows [chunk*256, chunk*256+256) or columns [chunk*64, chunk*64+64)
    int32_t kind;   // 0 = rows (r, R), 1 = columns (c, C)
    int32_t pad_;
};

// Per-tensor scalars produced by the finalize kernels, consumed by the sweeps.
struct TensorScalars {
    float sqrt_sum_r;   // sqrt(1^T r_t)
    float kappa;        // 1 / max(1, RMS(u_t)/d)                     (Eq. 1)
    float sqrt_sum_R;   // sqrt(1^T R_t)
    float rms_u;        // RMS(u_t), kept for inspection
    uint32_t pad_[4];
};
static_assert(sizeof(TensorScalars) == 32, "TensorScalars layout");

// Matrix tiles are launched per kernel variant so that each variant gets its own
// register allocation: gradient dtype x (vector loads | element-wise loads) x momentum dtype.
// Bit 0: binary32 gradient, bit 1: unaligned rows, bit 2: bfloat16 momentum.
constexpr int kVariants = 8;
inline int variant_of(int32_t flags)
{
    return ((flags & kFlagBf16Grad) ? 0 : 1) + ((flags & kFlagAligned) ? 0 : 2) +
           ((flags & kFlagBf16Momentum) ? 4 : 0);
}

// Consecutive tensors launched together: each phase is one launch per group and
// variant present.  Work items of a group: matrix tiles sorted by variant, then vectors.
struct Group {
    int32_t tensor_begin, tensor_end;
    int32_t var_begin[kVariants], var_end[kVariants];  // matrix tiles of each variant (sweeps 1 and 2)
    int32_t var3_begin[kVariants], var3_end[kVariants];  // the same matrices cut into the update sweep's tiles
    int32_t vec_begin, vec_end;                        // whole-vector items (one workgroup each)
    int32_t lvec_begin, lvec_end;                      // chunks of long vectors (two passes)
    int32_t fin_begin, fin_end;
    // tiles of the matrices on the on-chip path, per variant (aligned variants only), matrix
    // after matrix in list order: one launch per variant present
    int32_t res_begin[kVariants], res_end[kVariants];
    bool vectors_with_resident;  // no streaming matrix in the group: the whole-vector items ride in the
                                 // first on-chip launch instead of the first sweep-3 launch
};

struct Plan {
    std::vector<came_tensor_desc> descs;
    std::vector<TensorMeta> metas;
    std::vector<WorkItem> items;
    std::vector<FinalizeItem> fins;
    std::vector<Group> groups;
    int32_t tile_rows = 0;
    int32_t tile_rows3 = 0;  // update sweep
    int32_t algo = 0;
    int32_t momentum_dtype = 0;
    // Sweep 2 walks the tiles backwards: it then starts on the momenta sweep 3 wrote last (still in
    // the 256 MB on-package cache, and dirty: read there instead of being written back first and
    // fetched again later) and ends on the momenta and gradients sweep 3 reads first (measured:
    // sweep 2 10 % faster on a 109M-parameter list, 3 % on 350M-parameter lists, no difference
    // at 6.7B).
    bool reverse_sweep2 = false;
    // Lists of which the 256 MB on-package cache holds a noticeable part (up to 2^29 parameters:
    // at least 6 % of theta and M).  The update sweep leaves the last 256 MB it wrote dirty in that
    // cache.  Normally sweep 2's momentum loads push them out (and sweep 2 waits for their
    // write-back); on such a list sweep 2 loads the momentum with streaming loads, which leave
    // them where they are, and the update sweep walks its tiles in the opposite direction from
    // step to step, so that it begins where it ended last time: on entries that are still in
    // the cache and are then overwritten there instead of having been written back in between.
    // Measured: -4 % per step at 1.1e8 parameters, -1 % at 3.5e8; at 6.7e9 the streaming momentum
    // loads alone cost sweep 2 9 %, hence the limit.  Same results either way.
    bool keep_tail_cached = false;
    int64_t n_matrices = 0, n_vectors = 0, total_elements = 0;
    int64_t n_resident = 0, resident_elements = 0;  // matrices on the on-chip path
    bool any_folded = false;                        // a tile of sweeps 1 and 2 may hold 2 tile_rows rows of a matrix
    int32_t resident_wait_us = 0;
    // state blob
    size_t state_bytes = 0;
    // scratch blob sections (byte offsets)
    size_t off_metas = 0, off_items = 0, off_fins = 0, off_scalars = 0, off_ptrs = 0;
    size_t off_sync = 0;        // ResidentSync[count + 1], directly behind the scalars (cleared with them);
                                // the last entry's first word is the device-side failure flag
    size_t off_regions = 0;     // kResidentGrid regions of kResidentRegionBytes (only with matrices on the on-chip path)
    size_t ptr_slot_bytes = 0;  // one slot: theta[count], grad[count], bf16 parameter copy[count] (entries may be null)
    size_t off_partials = 0;
    size_t scratch_bytes = 0;
};

constexpr int kPtrSlots = 4;
constexpr int kPtrArrays = 3;

// Validates descs/opts and fills `plan`.  Returns CAME_OK or CAME_EINVAL.
int build_plan(const came_tensor_desc* descs, int32_t count, const came_options* opts, Plan* plan);

int validate_hyper(const came_hyper* h, double lr, int64_t step);

}  // namespace came
