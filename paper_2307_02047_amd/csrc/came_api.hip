// C ABI of the library (declared in include/came.h): validation, plan upload,
// per-step pointer table and the launch sequence.  Host code only; the kernels
// are in came_kernels.hip.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "came.h"
#include "came_kernels.h"
#include "came_plan.h"

using namespace came;

struct came_ctx {
    Plan plan;
    char* scratch = nullptr;  // caller's scratch blob (device)
    float* state = nullptr;   // caller's state blob (device)
    // pinned host staging for the per-step pointer table, one region per slot
    char* pinned = nullptr;
    int32_t* fail_host = nullptr;  // inside `pinned`: set by the on-chip kernel when a wait ran out
    hipEvent_t slot_event[kPtrSlots] = {};
    bool slot_used[kPtrSlots] = {};
    int slot = -1;
    std::vector<const void*> cached;  // theta[count], grad[count], bf16 copy[count] of the current slot
    int last_hip = 0;
    int64_t last_step = 0;
    int64_t steps_enqueued = 0;
    // phase timer
    bool profiling = false;
    struct Timed { hipEvent_t start, stop; int phase; };
    std::vector<Timed> timed;
};

namespace {

inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int hip_fail(came_ctx* ctx, hipError_t e)
{
    if (ctx) ctx->last_hip = static_cast<int>(e);
    return CAME_EHIP;
}

constexpr size_t kMaxTimed = 65536;

// Runs `launch` on stream s, bracketed by timing events when the phase timer is on.
template <class F>
hipError_t timed_launch(came_ctx* ctx, int phase, hipStream_t s, F launch)
{
    if (!ctx || !ctx->profiling || ctx->timed.size() >= kMaxTimed) return launch();
    came_ctx::Timed t{};
    t.phase = phase;
    hipError_t e = hipEventCreate(&t.start);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&t.stop);
    if (e != hipSuccess) { (void)hipEventDestroy(t.start); return e; }
    e = hipEventRecord(t.start, s);
    if (e == hipSuccess) e = launch();
    if (e == hipSuccess) e = hipEventRecord(t.stop, s);
    if (e != hipSuccess) { (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); return e; }
    ctx->timed.push_back(t);
    return hipSuccess;
}

constexpr uint64_t kTicksPerMicrosecond = 100;  // the constant clock the on-chip kernel times its waits with
constexpr int32_t kDefaultResidentWaitUs = 2000000;

// Where the on-chip kernel reports a wait that ran out, and how long it may wait.
ResidentCtl resident_ctl(const Plan& p, char* scratch, int32_t* fail_host)
{
    ResidentCtl c{};
    c.fail_dev = reinterpret_cast<int32_t*>(scratch + p.off_sync + sizeof(ResidentSync) * p.descs.size());
    c.fail_host = fail_host;
    c.regions = scratch + p.off_regions;
    c.limit_ticks = kTicksPerMicrosecond * static_cast<uint64_t>(p.resident_wait_us > 0 ? p.resident_wait_us : kDefaultResidentWaitUs);
    return c;
}

// Device-side views of a plan's tables inside a scratch blob, with pointer-table slot `slot`.
DeviceTables tables_in(const Plan& p, char* scratch, float* state, int slot)
{
    DeviceTables t{};
    t.metas = reinterpret_cast<const TensorMeta*>(scratch + p.off_metas);
    t.items = reinterpret_cast<const WorkItem*>(scratch + p.off_items);
    t.fins = reinterpret_cast<const FinalizeItem*>(scratch + p.off_fins);
    t.scalars = reinterpret_cast<TensorScalars*>(scratch + p.off_scalars);
    char* slot_base = scratch + p.off_ptrs + p.ptr_slot_bytes * static_cast<size_t>(slot);
    t.theta = reinterpret_cast<void* const*>(slot_base);
    t.grad = reinterpret_cast<const void* const*>(slot_base + sizeof(void*) * p.descs.size());
    t.theta16 = reinterpret_cast<void* const*>(slot_base + sizeof(void*) * 2 * p.descs.size());
    t.state = state;
    t.scratch = scratch;
    return t;
}

DeviceTables tables_for(const came_ctx* ctx, int slot)
{
    return tables_in(ctx->plan, ctx->scratch, ctx->state, slot);
}

// The caller's buffers must not overlap anything that is written: a parameter (or its
// bfloat16 copy) may overlap no other buffer and neither blob; gradients are only read,
// so two tensors may share one.  Sorted sweep over the address ranges.
int check_overlaps(const Plan& p, const void* state, const void* scratch, size_t scratch_bytes,
                   void* const* theta_dev, const void* const* grad_dev, void* const* theta16_dev)
{
    struct Range { uintptr_t lo, hi; bool written; };
    const size_t count = p.descs.size();
    std::vector<Range> r;
    r.reserve(3 * count + 2);
    auto add = [&](const void* ptr, size_t bytes, bool written) {
        const uintptr_t lo = reinterpret_cast<uintptr_t>(ptr);
        r.push_back(Range{lo, lo + bytes, written});
    };
    for (size_t t = 0; t < count; ++t) {
        const size_t nm = static_cast<size_t>(p.metas[t].n) * static_cast<size_t>(p.metas[t].m);
        add(theta_dev[t], nm * sizeof(float), true);
        if (grad_dev) add(grad_dev[t], nm * ((p.metas[t].flags & kFlagBf16Grad) ? 2 : 4), false);
        if (theta16_dev && theta16_dev[t]) add(theta16_dev[t], nm * 2, true);
    }
    add(state, p.state_bytes, true);
    add(scratch, scratch_bytes, true);
    std::sort(r.begin(), r.end(), [](const Range& a, const Range& b) { return a.lo < b.lo; });
    uintptr_t end_written = 0, end_any = 0;  // furthest end among the ranges already passed
    for (const Range& x : r) {
        if (x.lo < end_written) return CAME_EINVAL;
        if (x.written && x.lo < end_any) return CAME_EINVAL;
        end_any = std::max(end_any, x.hi);
        if (x.written) end_written = std::max(end_written, x.hi);
    }
    return CAME_OK;
}

// Pointer table: re-uploaded only when an address changed since the last call.
// theta16_dev may be null (no bf16 copies at all) or hold null entries.  check_grads: the
// gradient entries are real buffers (the placement probe fills them with placeholders).
int upload_pointers(came_ctx* ctx, void* const* theta_dev, const void* const* grad_dev,
                    void* const* theta16_dev, hipStream_t s, bool check_grads = true)
{
    const Plan& p = ctx->plan;
    const size_t count = p.descs.size();
    auto copy_of = [&](size_t t) -> const void* { return theta16_dev ? theta16_dev[t] : nullptr; };
    bool changed = ctx->slot < 0 || ctx->cached.size() != kPtrArrays * count;
    if (!changed) {
        for (size_t t = 0; t < count && !changed; ++t)
            changed = ctx->cached[t] != theta_dev[t] || ctx->cached[count + t] != grad_dev[t] ||
                      ctx->cached[2 * count + t] != copy_of(t);
    }
    if (changed) {
        // A new table means a host wait for a free slot and a copy out of a staging buffer that
        // later calls overwrite: neither may be recorded into a graph.
        hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
        const hipError_t ce = hipStreamIsCapturing(s, &capturing);
        if (ce != hipSuccess) return hip_fail(ctx, ce);
        if (capturing != hipStreamCaptureStatusNone) return CAME_EINVAL;
        const int rc = check_overlaps(ctx->plan, ctx->state, ctx->scratch, ctx->plan.scratch_bytes, theta_dev,
                                      check_grads ? grad_dev : nullptr, theta16_dev);
        if (rc != CAME_OK) return rc;
        const int slot = (ctx->slot + 1) % kPtrSlots;
        if (ctx->slot_used[slot]) {
            const hipError_t e = hipEventSynchronize(ctx->slot_event[slot]);
            if (e != hipSuccess) return hip_fail(ctx, e);
        }
        ctx->cached.resize(kPtrArrays * count);
        for (size_t t = 0; t < count; ++t) {
            ctx->cached[t] = theta_dev[t];
            ctx->cached[count + t] = grad_dev[t];
            ctx->cached[2 * count + t] = copy_of(t);
        }
        const size_t bytes = sizeof(void*) * kPtrArrays * count;
        char* host_slot = ctx->pinned + p.ptr_slot_bytes * static_cast<size_t>(slot);
        std::memcpy(host_slot, ctx->cached.data(), bytes);
        hipError_t e = hipMemcpyAsync(ctx->scratch + p.off_ptrs + p.ptr_slot_bytes * static_cast<size_t>(slot),
                                      host_slot, bytes, hipMemcpyHostToDevice, s);
        if (e != hipSuccess) { ctx->slot = -1; return hip_fail(ctx, e); }
        e = hipEventRecord(ctx->slot_event[slot], s);
        if (e != hipSuccess) { ctx->slot = -1; return hip_fail(ctx, e); }
        ctx->slot_used[slot] = true;
        ctx->slot = slot;
    }
    return CAME_OK;
}

// Host allocations inside the library (std::vector, new) may throw; nothing may leave through
// the C boundary.
template <class F>
int guarded(F body) noexcept
{
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return CAME_ENOMEM;
    } catch (...) {
        return CAME_EINVAL;
    }
}

// ---------------------------------------------------------------- library-owned scratch
//
// came_step_noalloc keeps its tables and partial sums in this array instead of a scratch blob
// of the caller's.  Every GPU that loads the library holds its own copy until the process
// ends.  In host code the name below is only a handle for hipGetSymbolAddress: the device
// address is resolved once per device and kept in static_scratch_ptr[]; every use on the
// host (kernel arguments, table pointers) goes through that pointer.
constexpr size_t kStaticScratchBytes = size_t(16) << 20;
constexpr int kMaxDevices = 64;
constexpr int32_t kNoallocMaxTensors = 64;
constexpr size_t kNoallocMaxTableBytes = size_t(256) << 10;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

char* static_scratch_ptr[kMaxDevices] = {};
std::mutex static_scratch_mutex;
thread_local int noalloc_last_hip = 0;

// Address of this device's copy of `scratch`, resolved at the first call on the device.
int static_scratch_of_current_device(char** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { noalloc_last_hip = static_cast<int>(e); return CAME_EHIP; }
    if (dev < 0 || dev >= kMaxDevices) return CAME_EINVAL;
    std::lock_guard<std::mutex> lock(static_scratch_mutex);
    if (!static_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) { noalloc_last_hip = static_cast<int>(e); return CAME_EHIP; }
        static_scratch_ptr[dev] = static_cast<char*>(ptr);
    }
    *out = static_scratch_ptr[dev];
    return CAME_OK;
}

// Host words -> device memory without a copy engine, a staging buffer or a wait: the words
// travel in the kernel's argument block (copied when the launch is enqueued), so the call is
// safe while a stream is being captured and the host buffer may be reused at once.
constexpr int kPokeWords = 768;  // 3 KiB of a 4 KiB argument block
struct PokeWords { uint32_t w[kPokeWords]; };

__global__ __launch_bounds__(256) void poke_kernel(uint32_t* dst, PokeWords words, int32_t count)
{
    for (int i = threadIdx.x; i < count; i += blockDim.x) dst[i] = words.w[i];
}

hipError_t poke(char* dst, const void* src, size_t bytes, hipStream_t s)
{
    const uint32_t* w = static_cast<const uint32_t*>(src);
    size_t left = bytes / sizeof(uint32_t);  // every table is a whole number of words
    uint32_t* d = reinterpret_cast<uint32_t*>(dst);
    while (left > 0) {
        const int32_t n = static_cast<int32_t>(std::min<size_t>(left, kPokeWords));
        PokeWords pw;
        std::memcpy(pw.w, w, sizeof(uint32_t) * n);
        poke_kernel<<<dim3(1), dim3(256), 0, s>>>(d, pw, n);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        w += n; d += n; left -= n;
    }
    return hipSuccess;
}

}  // namespace

extern "C" {

int came_state_size(const came_tensor_desc* descs, int32_t count, const came_options* opts,
                    size_t* state_bytes, size_t* scratch_bytes)
{
    return guarded([&]() -> int {
        if (!state_bytes || !scratch_bytes) return CAME_EINVAL;
        Plan plan;
        const int rc = build_plan(descs, count, opts, &plan);
        if (rc != CAME_OK) return rc;
        *state_bytes = plan.state_bytes;
        *scratch_bytes = plan.scratch_bytes;
        return CAME_OK;
    });
}

int came_plan_query(const came_tensor_desc* descs, int32_t count, const came_options* opts,
                    int64_t out[8])
{
    return guarded([&]() -> int {
        if (!out) return CAME_EINVAL;
        Plan plan;
        const int rc = build_plan(descs, count, opts, &plan);
        if (rc != CAME_OK) return rc;
        int64_t tiles = 0;  // the update sweep's own cut of the same matrices is not counted again
        for (const WorkItem& it : plan.items) tiles += it.kind != 4 && it.kind != 5;  // (kind 6 is a tile of sweeps 1 and 2)
        out[0] = plan.tile_rows;
        out[1] = kTileCols;
        out[2] = tiles;
        out[3] = static_cast<int64_t>(plan.fins.size());
        out[4] = static_cast<int64_t>(plan.groups.size());
        out[5] = plan.n_matrices;
        out[6] = plan.n_vectors;
        out[7] = plan.total_elements;
        return CAME_OK;
    });
}

double came_algorithmic_bytes(int32_t grad_bytes, int32_t momentum_bytes, int32_t algo, int32_t which)
{
    if ((grad_bytes != 2 && grad_bytes != 4) || (momentum_bytes != 2 && momentum_bytes != 4)) return 0.0;
    if (algo != CAME_ALGO_CAME && algo != CAME_ALGO_ADAFACTOR) return 0.0;
    const double g = static_cast<double>(grad_bytes), mb = static_cast<double>(momentum_bytes);
    const double s1 = g;                                          // read g
    const double s2 = g + (algo == CAME_ALGO_CAME ? mb : 0.0);    // read g (and M)
    const double s3 = g + 2.0 * mb + 8.0;                         // read g, M, theta; write M, theta
    if (which == 4) return algo == CAME_ALGO_CAME ? s3 : 0.0;     // on-chip path: every array crosses once
    switch (which) {
        case 0: return s1 + s2 + s3;
        case 1: return s1;
        case 2: return s2;
        case 3: return s3;
        default: return 0.0;
    }
}

int came_init_state(came_ctx** out, const came_tensor_desc* descs, int32_t count,
                    const came_options* opts, void* state_dev, size_t state_bytes,
                    void* scratch_dev, size_t scratch_bytes, void* hip_stream)
{
    return guarded([&]() -> int {
        if (!out) return CAME_EINVAL;
        *out = nullptr;
        if (!state_dev || !scratch_dev) return CAME_EINVAL;
        // owned here until handed over: every early return (and a throwing allocation) releases
        // the events, the pinned staging memory and the context itself through came_destroy
        std::unique_ptr<came_ctx, void (*)(came_ctx*)> owner(new (std::nothrow) came_ctx(), came_destroy);
        came_ctx* ctx = owner.get();
        if (!ctx) return CAME_ENOMEM;
        int rc = build_plan(descs, count, opts, &ctx->plan);
        if (rc != CAME_OK) return rc;
        const Plan& p = ctx->plan;
        if (state_bytes < p.state_bytes || scratch_bytes < p.scratch_bytes) return CAME_ESIZE;
        if (!aligned_to(state_dev, 256) || !aligned_to(scratch_dev, 256)) return CAME_EALIGN;
        ctx->state = static_cast<float*>(state_dev);
        ctx->scratch = static_cast<char*>(scratch_dev);
        hipStream_t s = static_cast<hipStream_t>(hip_stream);

        hipError_t e = hipSuccess;
        if (p.n_resident > 0) {
            // the on-chip path counts on all kResidentGrid workgroups being on the chip at once: the
            // plan, made without a device, is checked here against what this device and this build give
            int dev = -1, cus = 0;
            e = hipGetDevice(&dev);
            if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
            if (e != hipSuccess) return CAME_EHIP;
            for (int v = 0; v < kVariants; ++v) {
                bool present = false;
                for (const Group& g : p.groups) present = present || g.res_end[v] > g.res_begin[v];
                if (!present) continue;
                int per_cu = 0;
                e = resident_occupancy(v, &per_cu);
                if (e != hipSuccess) return CAME_EHIP;
                if (static_cast<int64_t>(per_cu) * cus < kResidentGrid) return CAME_EHIP;
            }
        }
        constexpr size_t kFlagBytes = 256;
        e = hipHostMalloc(reinterpret_cast<void**>(&ctx->pinned), p.ptr_slot_bytes * kPtrSlots + kFlagBytes, hipHostMallocDefault);
        if (e != hipSuccess) { ctx->pinned = nullptr; return CAME_EHIP; }
        ctx->fail_host = reinterpret_cast<int32_t*>(ctx->pinned + p.ptr_slot_bytes * kPtrSlots);
        *ctx->fail_host = 0;
        for (int k = 0; k < kPtrSlots; ++k) {
            e = hipEventCreateWithFlags(&ctx->slot_event[k], hipEventDisableTiming);
            if (e != hipSuccess) { ctx->slot_event[k] = nullptr; return CAME_EHIP; }
        }

        // plan tables -> scratch (synchronous copies from pageable memory), then zero the
        // per-tensor scalars/counters and the optimizer state with fill kernels
        e = hipMemcpy(ctx->scratch + p.off_metas, p.metas.data(), sizeof(TensorMeta) * p.metas.size(), hipMemcpyHostToDevice);
        if (e != hipSuccess) return CAME_EHIP;
        if (!p.items.empty()) {
            e = hipMemcpy(ctx->scratch + p.off_items, p.items.data(), sizeof(WorkItem) * p.items.size(), hipMemcpyHostToDevice);
            if (e != hipSuccess) return CAME_EHIP;
        }
        if (!p.fins.empty()) {
            e = hipMemcpy(ctx->scratch + p.off_fins, p.fins.data(), sizeof(FinalizeItem) * p.fins.size(), hipMemcpyHostToDevice);
            if (e != hipSuccess) return CAME_EHIP;
        }
        // (the counters of the on-chip path and its failure flag lie directly behind the scalars)
        e = launch_fill_zero_bytes(ctx->scratch + p.off_scalars,
                                   p.off_sync + sizeof(ResidentSync) * (p.descs.size() + 1) - p.off_scalars, s);
        if (e != hipSuccess) return CAME_EHIP;
        e = launch_fill_zero(ctx->state, p.state_bytes / sizeof(float), s);
        if (e != hipSuccess) return CAME_EHIP;
        owner.release();
        *out = ctx;
        return CAME_OK;
    });
}

// Argument checks shared by every step entry point: hyper-parameters, pointers, alignment.
static int check_step_arguments(const Plan& p, void* const* theta_dev, const void* const* grad_dev,
                                void* const* theta16_dev, const came_hyper* hyper, double lr, int64_t step)
{
    if (!theta_dev || !grad_dev) return CAME_EINVAL;
    const int rc = validate_hyper(hyper, lr, step);
    if (rc != CAME_OK) return rc;
    const size_t count = p.descs.size();
    for (size_t t = 0; t < count; ++t) {
        if (!theta_dev[t] || !grad_dev[t]) return CAME_EINVAL;
        if (!aligned_to(theta_dev[t], 16) || !aligned_to(grad_dev[t], 16)) return CAME_EALIGN;
        if (theta_dev[t] == grad_dev[t]) return CAME_EINVAL;
        if (theta16_dev && theta16_dev[t]) {
            if (!aligned_to(theta16_dev[t], 16)) return CAME_EALIGN;
            if (theta16_dev[t] == theta_dev[t] || theta16_dev[t] == grad_dev[t]) return CAME_EINVAL;
        }
    }
    return CAME_OK;
}

// The launch sequence of one step over the plan's groups, on tables that are already in device
// memory.  ctx (may be null) only serves the phase timer and the record of a failed HIP call.
// odd_step: whether this is an odd-numbered call on its context (lists small against the
// on-package cache alternate the update sweep's direction, see Plan::keep_tail_cached).
static int enqueue_step(came_ctx* ctx, const Plan& p, const DeviceTables& tb, const came_hyper* hyper,
                        double lr, hipStream_t s, int* hip_error, const ResidentCtl* rctl = nullptr,
                        bool odd_step = false)
{
    const bool reverse3 = p.keep_tail_cached && odd_step;
    auto failed = [&](hipError_t e) {
        if (hip_error) *hip_error = static_cast<int>(e);
        return hip_fail(ctx, e);
    };
    SweepHyper sh{};
    sh.beta1 = static_cast<float>(hyper->beta1);
    sh.one_minus_beta1 = static_cast<float>(1.0 - hyper->beta1);
    sh.beta2 = static_cast<float>(hyper->beta2);
    sh.one_minus_beta2 = static_cast<float>(1.0 - hyper->beta2);
    sh.beta3 = static_cast<float>(hyper->beta3);
    sh.one_minus_beta3 = static_cast<float>(1.0 - hyper->beta3);
    sh.eps1 = static_cast<float>(hyper->eps1);
    sh.eps2 = static_cast<float>(hyper->eps2);
    sh.lr = static_cast<float>(lr);
    sh.decay = static_cast<float>(1.0 - lr * hyper->weight_decay);
    sh.algo = p.algo;
    FinalizeHyper fh{};
    fh.beta1 = hyper->beta1;
    fh.beta2 = hyper->beta2;
    fh.one_minus_beta2 = 1.0 - hyper->beta2;
    fh.beta3 = hyper->beta3;
    fh.one_minus_beta3 = 1.0 - hyper->beta3;
    fh.eps1 = hyper->eps1;
    fh.eps2 = hyper->eps2;
    fh.clip_d = hyper->clip_d;
    fh.algo = p.algo;

    for (const Group& g : p.groups) {
        hipError_t e = hipSuccess;
        if (g.lvec_end > g.lvec_begin) {
            e = timed_launch(ctx, 5, s, [&] { return launch_long_vectors(tb, g.lvec_begin, g.lvec_end, sh, fh, s); });
            if (e != hipSuccess) return failed(e);
        }
        const int32_t lds_rows = p.any_folded ? 2 * p.tile_rows : p.tile_rows;
        bool on_chip = false;
        for (int v = 0; v < kVariants; ++v) on_chip = on_chip || g.res_end[v] > g.res_begin[v];
        if (on_chip) {
            if (!rctl) return CAME_EINVAL;  // an entry point without a failure channel planned the on-chip path
            bool vectors_ride = g.vectors_with_resident;
            for (int v = 0; v < kVariants; ++v) {
                if (g.res_end[v] == g.res_begin[v]) continue;
                const int32_t vb = vectors_ride ? g.vec_begin : 0, ve = vectors_ride ? g.vec_end : 0;
                e = timed_launch(ctx, 6, s, [&] { return launch_resident(tb, v, g.res_begin[v], g.res_end[v], vb, ve, sh, fh, *rctl, s); });
                if (e != hipSuccess) return failed(e);
                vectors_ride = false;
            }
        }
        if (g.fin_end == g.fin_begin) {  // no streaming matrix
            if (!g.vectors_with_resident && g.vec_end > g.vec_begin) {
                e = timed_launch(ctx, 5, s, [&] { return launch_vectors(tb, g.vec_begin, g.vec_end, sh, fh, s); });
                if (e != hipSuccess) return failed(e);
            }
            continue;
        }
        for (int v = 0; v < kVariants; ++v) {
            if (g.var_end[v] == g.var_begin[v]) continue;
            e = timed_launch(ctx, 0, s, [&] { return launch_sweep1(tb, v, lds_rows, g.var_begin[v], g.var_end[v], s); });
            if (e != hipSuccess) return failed(e);
        }
        e = timed_launch(ctx, 1, s, [&] { return launch_finalize1(tb, g.fin_begin, g.fin_end, fh, s); });
        if (e != hipSuccess) return failed(e);
        for (int v = 0; v < kVariants; ++v) {
            if (g.var_end[v] == g.var_begin[v]) continue;
            e = timed_launch(ctx, 2, s, [&] { return launch_sweep2(tb, v, p.algo, lds_rows, g.var_begin[v], g.var_end[v], p.reverse_sweep2, p.keep_tail_cached, s); });
            if (e != hipSuccess) return failed(e);
        }
        e = timed_launch(ctx, 3, s, [&] { return launch_finalize2(tb, g.fin_begin, g.fin_end, fh, s); });
        if (e != hipSuccess) return failed(e);
        // the whole-vector items are the first workgroups of the first sweep-3 launch: independent,
        // latency-bound work that is over long before the launch's tiles are
        bool vectors_pending = g.vec_end > g.vec_begin;
        for (int v = 0; v < kVariants; ++v) {
            if (g.var_end[v] == g.var_begin[v]) continue;
            const int32_t vb = vectors_pending ? g.vec_begin : 0, ve = vectors_pending ? g.vec_end : 0;
            e = timed_launch(ctx, 4, s, [&] { return launch_sweep3(tb, v, p.tile_rows3, g.var3_begin[v], g.var3_end[v], vb, ve, reverse3, sh, fh, s); });
            if (e != hipSuccess) return failed(e);
            vectors_pending = false;
        }
    }
    return CAME_OK;
}

static int step_impl(came_ctx* ctx, void* const* theta_dev, const void* const* grad_dev,
                     void* const* theta16_dev, const came_hyper* hyper, double lr, int64_t step,
                     void* hip_stream)
{
    if (!ctx) return CAME_EINVAL;
    if (*static_cast<volatile int32_t*>(ctx->fail_host) != 0) return CAME_ETIMEOUT;
    int rc = check_step_arguments(ctx->plan, theta_dev, grad_dev, theta16_dev, hyper, lr, step);
    if (rc != CAME_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    rc = upload_pointers(ctx, theta_dev, grad_dev, theta16_dev, s);
    if (rc != CAME_OK) return rc;
    const ResidentCtl rctl = resident_ctl(ctx->plan, ctx->scratch, ctx->fail_host);
    rc = enqueue_step(ctx, ctx->plan, tables_for(ctx, ctx->slot), hyper, lr, s, nullptr, &rctl, (ctx->steps_enqueued++ & 1) != 0);
    if (rc != CAME_OK) return rc;
    ctx->last_step = step;
    return CAME_OK;
}

int came_step(came_ctx* ctx, void* const* theta_dev, const void* const* grad_dev,
              const came_hyper* hyper, double lr, int64_t step, void* hip_stream)
{
    return guarded([&]() -> int {
        return step_impl(ctx, theta_dev, grad_dev, nullptr, hyper, lr, step, hip_stream);
    });
}

int came_step_bf16_copy(came_ctx* ctx, void* const* theta_dev, const void* const* grad_dev,
                        void* const* theta_bf16_dev, const came_hyper* hyper, double lr, int64_t step,
                        void* hip_stream)
{
    return guarded([&]() -> int {
        if (!theta_bf16_dev) return CAME_EINVAL;
        return step_impl(ctx, theta_dev, grad_dev, theta_bf16_dev, hyper, lr, step, hip_stream);
    });
}

int came_step_noalloc(const came_tensor_desc* descs, int32_t count, const came_options* opts,
                      void* state_dev, size_t state_bytes, int32_t zero_state, void* const* theta_dev,
                      const void* const* grad_dev, const came_hyper* hyper, double lr, int64_t step,
                      void* hip_stream)
{
    return guarded([&]() -> int {
        if (!state_dev || count > kNoallocMaxTensors) return !state_dev ? CAME_EINVAL : CAME_ESIZE;
        // no context, hence nowhere for the on-chip kernel to report a wait that ran out: streaming only
        came_options o{};
        if (opts) o = *opts;
        if (o.resident == CAME_RESIDENT_ON) return CAME_EINVAL;
        o.resident = CAME_RESIDENT_OFF;
        Plan p;  // host memory only
        int rc = build_plan(descs, count, &o, &p);
        if (rc != CAME_OK) return rc;
        const size_t table_bytes = sizeof(TensorMeta) * p.metas.size() + sizeof(WorkItem) * p.items.size() +
                                   sizeof(FinalizeItem) * p.fins.size() + sizeof(void*) * kPtrArrays * p.descs.size();
        if (p.scratch_bytes > kStaticScratchBytes || table_bytes > kNoallocMaxTableBytes) return CAME_ESIZE;
        if (state_bytes < p.state_bytes) return CAME_ESIZE;
        if (!aligned_to(state_dev, 256)) return CAME_EALIGN;
        rc = check_step_arguments(p, theta_dev, grad_dev, nullptr, hyper, lr, step);
        if (rc != CAME_OK) return rc;
        char* sp = nullptr;
        rc = static_scratch_of_current_device(&sp);
        if (rc != CAME_OK) return rc;
        rc = check_overlaps(p, state_dev, sp, kStaticScratchBytes, theta_dev, grad_dev, nullptr);
        if (rc != CAME_OK) return rc;

        hipStream_t s = static_cast<hipStream_t>(hip_stream);
        auto failed = [&](hipError_t e) { noalloc_last_hip = static_cast<int>(e); return CAME_EHIP; };
        // tables of this call; the array still holds the previous call's
        hipError_t e = poke(sp + p.off_metas, p.metas.data(), sizeof(TensorMeta) * p.metas.size(), s);
        if (e == hipSuccess && !p.items.empty()) e = poke(sp + p.off_items, p.items.data(), sizeof(WorkItem) * p.items.size(), s);
        if (e == hipSuccess && !p.fins.empty()) e = poke(sp + p.off_fins, p.fins.data(), sizeof(FinalizeItem) * p.fins.size(), s);
        if (e != hipSuccess) return failed(e);
        {
            // pointer table, slot 0: theta[count], grad[count], no bfloat16 copies
            const void* ptrs[kPtrArrays * kNoallocMaxTensors] = {};
            for (int32_t t = 0; t < count; ++t) {
                ptrs[t] = theta_dev[t];
                ptrs[count + t] = grad_dev[t];
            }
            e = poke(sp + p.off_ptrs, ptrs, sizeof(void*) * kPtrArrays * count, s);
            if (e != hipSuccess) return failed(e);
        }
        // what came_init_state clears: the per-tensor scalars, and the state when asked to
        e = launch_fill_zero_bytes(sp + p.off_scalars, sizeof(TensorScalars) * p.descs.size(), s);
        if (e == hipSuccess && zero_state) e = launch_fill_zero(static_cast<float*>(state_dev), p.state_bytes / sizeof(float), s);
        if (e != hipSuccess) return failed(e);
        return enqueue_step(nullptr, p, tables_in(p, sp, static_cast<float*>(state_dev), 0), hyper, lr, s, &noalloc_last_hip, nullptr, (step & 1) != 0);
    });
}

int came_plan_traffic(const came_tensor_desc* descs, int32_t count, const came_options* opts, double out[4])
{
    return guarded([&]() -> int {
        if (!out) return CAME_EINVAL;
        Plan plan;
        const int rc = build_plan(descs, count, opts, &plan);
        if (rc != CAME_OK) return rc;
        const int32_t mb = plan.momentum_dtype == CAME_MOMENTUM_BF16 ? 2 : 4;
        double planned = 0.0, streaming = 0.0;
        for (const TensorMeta& tm : plan.metas) {
            const int32_t gb = (tm.flags & kFlagBf16Grad) ? 2 : 4;
            const double nm = static_cast<double>(tm.n) * static_cast<double>(tm.m);
            if (tm.flags & kFlagVector) {
                // g read; v, s, theta and M read and written; vectors too long for one workgroup read g and v twice
                const double per = 24.0 + gb + 2.0 * mb + (tm.n > kFusedVectorMax ? gb + 4.0 : 0.0);
                planned += per * nm;
                streaming += per * nm;
                continue;
            }
            const double stream_per = came_algorithmic_bytes(gb, mb, plan.algo, 0);
            streaming += stream_per * nm;
            planned += ((tm.flags & kFlagResident) ? came_algorithmic_bytes(gb, mb, plan.algo, 4) : stream_per) * nm;
        }
        out[0] = static_cast<double>(plan.n_resident);
        out[1] = static_cast<double>(plan.resident_elements);
        out[2] = planned;
        out[3] = streaming;
        return CAME_OK;
    });
}

int came_device_status(came_ctx* ctx, void* hip_stream)
{
    if (!ctx) return CAME_EINVAL;
    const hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return hip_fail(ctx, e);
    return *static_cast<volatile int32_t*>(ctx->fail_host) != 0 ? CAME_ETIMEOUT : CAME_OK;
}

int came_state_view_get(const came_ctx* ctx, int32_t i, came_state_view* view)
{
    if (!ctx || !view) return CAME_EINVAL;
    if (i < 0 || static_cast<size_t>(i) >= ctx->plan.metas.size()) return CAME_EINVAL;
    const TensorMeta& tm = ctx->plan.metas[i];
    view->m = ctx->state + tm.off_M;
    view->r = ctx->state + tm.off_r;
    view->R = ctx->state + tm.off_R;
    view->c = tm.off_c >= 0 ? ctx->state + tm.off_c : nullptr;
    view->C = tm.off_C >= 0 ? ctx->state + tm.off_C : nullptr;
    return CAME_OK;
}

int came_probe_placement(came_ctx* ctx, void* const* theta_dev, const void* const* grad_dev,
                         void* hip_stream, int32_t repeats, double* gbytes_per_s)
{
    return guarded([&]() -> int {
        if (!ctx || !theta_dev || !gbytes_per_s || repeats < 1 || repeats > 1000) return CAME_EINVAL;
        const Plan& p = ctx->plan;
        const size_t count = p.descs.size();
        for (size_t t = 0; t < count; ++t) {
            if (!theta_dev[t]) return CAME_EINVAL;
            if (!aligned_to(theta_dev[t], 16)) return CAME_EALIGN;
            if (grad_dev) {
                if (!grad_dev[t]) return CAME_EINVAL;
                if (!aligned_to(grad_dev[t], 16)) return CAME_EALIGN;
            }
        }
        *gbytes_per_s = 0.0;
        hipStream_t s = static_cast<hipStream_t>(hip_stream);
        // without gradients the pointer table's gradient half just repeats theta (never read)
        std::vector<const void*> fake(theta_dev, theta_dev + count);
        int rc = upload_pointers(ctx, theta_dev, grad_dev ? grad_dev : fake.data(), nullptr, s, grad_dev != nullptr);
        if (rc != CAME_OK) return rc;
        ctx->cached.clear();  // force a fresh table at the next came_step
        const int used_slot = ctx->slot;
        const bool with_g = grad_dev != nullptr;
        double bytes = 0.0;
        // every streamed matrix with 16-byte aligned rows, all of its entries
        for (const TensorMeta& tm : p.metas) {
            if ((tm.flags & (kFlagVector | kFlagResident)) || !(tm.flags & kFlagAligned)) continue;
            const double mb = (tm.flags & kFlagBf16Momentum) ? 2.0 : 4.0;
            const double gb = (tm.flags & kFlagBf16Grad) ? 2.0 : 4.0;
            // sweep 3's streams: theta and M read and written (g read);
            // with gradients also sweep 2's: g and M read
            double per = 8.0 + 2.0 * mb;
            if (with_g) per += gb + (gb + mb);
            bytes += per * static_cast<double>(tm.n) * static_cast<double>(tm.m);
        }
        if (bytes == 0.0) return CAME_OK;
        const DeviceTables tb = tables_for(ctx, used_slot);
        hipEvent_t e0, e1;
        hipError_t e = hipEventCreate(&e0);
        if (e != hipSuccess) return hip_fail(ctx, e);
        e = hipEventCreate(&e1);
        if (e != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(ctx, e); }
        auto run_once = [&]() -> hipError_t {
            for (int mode = with_g ? 1 : 0; mode >= 0; --mode)
                for (const Group& g : p.groups)
                    for (int v = 0; v < kVariants; ++v) {
                        if (v & 2) continue;
                        // the update sweep's streams in its own tiles, sweep 2's in the shared ones
                        const hipError_t le = mode == 0 ? launch_placement_probe(tb, g.var3_begin[v], g.var3_end[v], mode, with_g, s)
                                                        : launch_placement_probe(tb, g.var_begin[v], g.var_end[v], mode, with_g, s);
                        if (le != hipSuccess) return le;
                    }
            return hipSuccess;
        };
        e = run_once();  // warm-up
        if (e == hipSuccess) e = hipEventRecord(e0, s);
        for (int r = 0; r < repeats && e == hipSuccess; ++r) e = run_once();
        if (e == hipSuccess) e = hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
        if (e != hipSuccess) return hip_fail(ctx, e);
        if (ms > 0.f) *gbytes_per_s = bytes * repeats / (static_cast<double>(ms) * 1e-3) / 1e9;
        return CAME_OK;
    });
}

int came_profile_enable(came_ctx* ctx, int32_t on)
{
    if (!ctx) return CAME_EINVAL;
    ctx->profiling = on != 0;
    return CAME_OK;
}

int came_profile_read(came_ctx* ctx, double phase_ms[7], int64_t phase_launches[7])
{
    return guarded([&]() -> int {
        if (!ctx || !phase_ms || !phase_launches) return CAME_EINVAL;
        for (int k = 0; k < 7; ++k) { phase_ms[k] = 0.0; phase_launches[k] = 0; }
        int rc = CAME_OK;
        for (const came_ctx::Timed& t : ctx->timed) {
            hipError_t e = hipEventSynchronize(t.stop);
            float ms = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, t.start, t.stop);
            if (e == hipSuccess) {
                phase_ms[t.phase] += static_cast<double>(ms);
                phase_launches[t.phase] += 1;
            } else {
                rc = hip_fail(ctx, e);
            }
            (void)hipEventDestroy(t.start);
            (void)hipEventDestroy(t.stop);
        }
        ctx->timed.clear();
        return rc;
    });
}

int came_last_hip_error(const came_ctx* ctx) { return ctx ? ctx->last_hip : noalloc_last_hip; }

void came_destroy(came_ctx* ctx)
{
    if (!ctx) return;
    for (const came_ctx::Timed& t : ctx->timed) {
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
    }
    for (int k = 0; k < kPtrSlots; ++k)
        if (ctx->slot_event[k]) (void)hipEventDestroy(ctx->slot_event[k]);
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    delete ctx;
}

const char* came_strerror(int status)
{
    switch (status) {
        case CAME_OK: return "ok";
        case CAME_EINVAL: return "invalid argument";
        case CAME_ESIZE: return "state or scratch blob too small";
        case CAME_EALIGN: return "device pointer not aligned as required";
        case CAME_EHIP: return "HIP runtime call failed";
        case CAME_ENOMEM: return "host allocation failed";
        case CAME_ETIMEOUT: return "a wait inside the on-chip kernel ran into its time limit";
        default: return "unknown status";
    }
}

}  // extern "C"
