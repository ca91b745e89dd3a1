// Launch wrappers of the gfx950 kernels (defined in came_kernels.hip).
#pragma once

#include <hip/hip_runtime_api.h>

#include "came_plan.h"

namespace came {

// Coefficients the sweep kernels use, rounded once from the caller's doubles.
struct SweepHyper {
    float beta1, one_minus_beta1;
    float beta2, one_minus_beta2;
    float beta3, one_minus_beta3;
    float eps1, eps2;
    float lr;
    float decay;  // 1 - eta * lambda (decoupled weight decay; 1 when there is none)
    int32_t algo;
};

// Coefficients the finalize kernels use (O(n+m) work, done in double).
struct FinalizeHyper {
    double beta1;
    double beta2, one_minus_beta2;
    double beta3, one_minus_beta3;
    double eps1, eps2;
    double clip_d;
    int32_t algo;
};

// Device-side views of the scratch sections plus the caller's state blob.
struct DeviceTables {
    const TensorMeta* metas;
    const WorkItem* items;
    const FinalizeItem* fins;
    TensorScalars* scalars;
    void* const* theta;        // current pointer slot: theta[count]
    const void* const* grad;   //                       grad[count]
    void* const* theta16;      //                       bf16 copy of theta[count]; null entries: no copy
    float* state;
    char* scratch;
};

// How the on-chip kernel reports a wait that ran into its limit.
struct ResidentCtl {
    int32_t* fail_dev;     // device memory (scratch blob): non-zero once any workgroup gave up a wait
    int32_t* fail_host;    // pinned host memory, device-accessible: the same, for the host to see
    uint64_t limit_ticks;  // longest single wait, in ticks of the constant 100 MHz clock
    char* regions;         // device memory (scratch blob): the workgroups' partial-sum regions
};

hipError_t launch_fill_zero(float* p, size_t count, hipStream_t s);
hipError_t launch_fill_zero_bytes(void* p, size_t bytes, hipStream_t s);

// `variant` (see variant_of) selects the kernel instantiation; all work items in
// [item_begin, item_end) must be matrix tiles of tensors of that variant.

// Memory traffic of a sweep over the matrix tiles [item_begin, item_end) without its arithmetic,
// contents unchanged.  mode 0: theta and M read and rewritten with their own bits (sweep 3),
// g read as well when with_g; mode 1: g and M read only (sweep 2; needs with_g).
hipError_t launch_placement_probe(const DeviceTables& t, int32_t item_begin, int32_t item_end, int mode,
                                  bool with_g, hipStream_t s);

// Complete Algorithm-2 update of the vectors [item_begin, item_end), one workgroup each.
hipError_t launch_vectors(const DeviceTables& t, int32_t item_begin, int32_t item_end,
                          const SweepHyper& h, const FinalizeHyper& fh, hipStream_t s);
// Complete update of the long-vector chunks [item_begin, item_end): two launches (second
// moment and chunk sums of u^2, then everything else).
hipError_t launch_long_vectors(const DeviceTables& t, int32_t item_begin, int32_t item_end,
                               const SweepHyper& h, const FinalizeHyper& fh, hipStream_t s);
// lds_rows (sweeps 1 and 2): rows of the matrix a tile can hold, which sizes the per-row buffers in
// LDS: the plan's tile_rows, twice that when the list has folded matrices.
// Sweep 1: row/column sums of g^2 of the matrix tiles [item_begin, item_end).
hipError_t launch_sweep1(const DeviceTables& t, int variant, int32_t lds_rows, int32_t item_begin,
                         int32_t item_end, hipStream_t s);
// Finalize 1: r, c and the per-workgroup sums of r.
hipError_t launch_finalize1(const DeviceTables& t, int32_t fin_begin, int32_t fin_end,
                            const FinalizeHyper& h, hipStream_t s);
// Sweep 2: row/column sums of u^2, u*M, M^2 and the per-tile sum of u^2 (Algorithm 1: the latter only).
// reverse: take the tiles last to first (same results; see Plan::reverse_sweep2).  stream_m: load
// the momentum with streaming loads as well (see Plan::keep_tail_cached).
hipError_t launch_sweep2(const DeviceTables& t, int variant, int32_t algo, int32_t lds_rows,
                         int32_t item_begin, int32_t item_end, bool reverse, bool stream_m, hipStream_t s);
// Finalize 2: kappa (Eq. 1), R, C and the per-workgroup sums of R.
hipError_t launch_finalize2(const DeviceTables& t, int32_t fin_begin, int32_t fin_end,
                            const FinalizeHyper& h, hipStream_t s);
// Sweep 3: momentum and parameter update.  The launch's first vec_end - vec_begin workgroups
// update the whole-vector items [vec_begin, vec_end) (pass 0, 0 for none).  reverse: take the
// tiles last to first (same results).
hipError_t launch_sweep3(const DeviceTables& t, int variant, int32_t tile_rows, int32_t item_begin,
                         int32_t item_end, int32_t vec_begin, int32_t vec_end, bool reverse, const SweepHyper& h,
                         const FinalizeHyper& fh, hipStream_t s);

// On-chip path (came_resident.hip): the complete Algorithm-2 step of the matrices whose tiles are
// the work items [item_begin, item_end) (kind 3, all of `variant`), one launch of at most
// kResidentGrid workgroups.  The whole-vector items [vec_begin, vec_end) ride along; pass an empty
// range for none.
hipError_t launch_resident(const DeviceTables& t, int variant, int32_t item_begin, int32_t item_end,
                           int32_t vec_begin, int32_t vec_end, const SweepHyper& h, const FinalizeHyper& fh,
                           const ResidentCtl& ctl, hipStream_t s);
// Workgroups of the on-chip kernel `variant` that the runtime will keep on one compute unit at once.
hipError_t resident_occupancy(int variant, int* workgroups_per_cu);

}  // namespace came
