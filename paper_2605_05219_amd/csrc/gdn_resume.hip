// C ABI of the library: argument validation, planning, plan upload and kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "gdn_host.h"
#include "gdn_plan.h"
#include "gdn_prep_kernel.h"
#include "gdn_decode_kernel.h"
#include "gdn_fused_kernel.h"
#include "gdn_probe_kernel.h"
#include "gdn_recur_kernel.h"
#include "gdn_resume.h"

namespace gdn {
namespace {

inline int32_t hip_err(hipError_t e) { return e == hipSuccess ? GDN_OK : GDN_ERR_HIP - (int32_t)e; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ------------------------------------------------------------------ checkpoint pool copies
constexpr int COPY_IDS = 256;   // slot ids carried by value per launch
constexpr int COPY_THREADS = 256;

struct CopyIds {
    int32_t id[COPY_IDS];
};

// blockIdx.y = state within the batch; a thread moves ONE 16-byte piece, a workgroup 4 KiB, with non-temporal accesses
// (nothing is read twice).  Measured on 1 GiB each way: 6.5 TB/s in this form against 5.4 TB/s for a grid of a few
// thousand workgroups that stride over the data with four loads in flight per thread: the memory system is fed best by
// very many small workgroups, each gone as soon as its one request is answered.
// GATHER: dst[y] = pool[id[y]] (zeros for id -1);  else pool[id[y]] = src[y].
template <bool GATHER>
__global__ void __launch_bounds__(COPY_THREADS) ckpt_copy_kernel(const f32x4* __restrict__ from, f32x4* __restrict__ to,
                                                                 int64_t from_stride4, int64_t to_stride4,
                                                                 int64_t n4, CopyIds ids) {
    const int y = blockIdx.y;
    const int32_t id = ids.id[y];
    const int64_t i = (int64_t)blockIdx.x * COPY_THREADS + threadIdx.x;
    if (i >= n4) return;
    const f32x4* src = GATHER ? from + (int64_t)id * from_stride4 : from + (int64_t)y * from_stride4;
    f32x4* dst = GATHER ? to + (int64_t)y * to_stride4 : to + (int64_t)id * to_stride4;
    if (GATHER && id < 0) {
        __builtin_nontemporal_store(f32x4{0.f, 0.f, 0.f, 0.f}, dst + i);
        return;
    }
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

int32_t check_copy_args(const void* pool, int64_t slot_stride, int32_t n_slots, const int32_t* ids, int32_t n,
                        const void* other, int64_t other_stride, int64_t state_elems, bool allow_minus_one) {
    if (n < 0 || n_slots < 0 || state_elems < 0) return GDN_ERR_COUNT;
    if (n == 0 || state_elems == 0) return GDN_OK;
    if (!pool || !ids || !other) return GDN_ERR_NULL;
    if (!aligned16(pool) || !aligned16(other)) return GDN_ERR_ALIGN;
    if ((state_elems & 3) || (slot_stride & 3) || (other_stride & 3)) return GDN_ERR_ALIGN;
    if (slot_stride < state_elems || other_stride < state_elems) return GDN_ERR_SHAPE;
    for (int32_t i = 0; i < n; ++i) {
        if (ids[i] >= n_slots) return GDN_ERR_SLOT_RANGE;
        if (ids[i] < (allow_minus_one ? -1 : 0)) return GDN_ERR_SLOT_RANGE;
    }
    return GDN_OK;
}

template <bool GATHER>
int32_t launch_copy(const float* from, float* to, int64_t from_stride, int64_t to_stride, int64_t state_elems,
                    const int32_t* ids, int32_t n, hipStream_t stream) {
    const int64_t n4 = state_elems / 4;
    const int64_t gx = (n4 + COPY_THREADS - 1) / COPY_THREADS;      // one 16-byte piece per thread
    if (gx > INT32_MAX) return GDN_ERR_COUNT;
    for (int32_t base = 0; base < n; base += COPY_IDS) {
        const int32_t m = std::min(COPY_IDS, n - base);
        CopyIds batch;
        std::memset(&batch, 0, sizeof batch);
        std::memcpy(batch.id, ids + base, sizeof(int32_t) * m);
        const dim3 grid((unsigned)gx, (unsigned)m);
        const f32x4* f = reinterpret_cast<const f32x4*>(from) + (GATHER ? 0 : (int64_t)base * (from_stride / 4));
        f32x4* t = reinterpret_cast<f32x4*>(to) + (GATHER ? (int64_t)base * (to_stride / 4) : 0);
        hipLaunchKernelGGL(ckpt_copy_kernel<GATHER>, grid, dim3(COPY_THREADS), 0, stream, f, t, from_stride / 4,
                           to_stride / 4, n4, batch);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_err(e);
    }
    return GDN_OK;
}

// ------------------------------------------------------------------ plan image without allocation or staging
// gdn_resume_prefill_static keeps its plan image in this array (one copy per GPU, held until the process ends)
// and writes it there by kernel arguments, so the call needs neither a workspace nor the pinned staging ring.
constexpr int64_t STATIC_SCRATCH_BYTES = 512 << 10;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int PLAN_PIECE_WORDS = 896;   // 3.5 KiB of the 4 KiB a launch may carry as arguments
struct PlanPiece {
    int32_t w[PLAN_PIECE_WORDS];
};
__global__ void __launch_bounds__(256) plan_write_kernel(PlanPiece piece, int32_t* __restrict__ dst, int32_t n) {
    for (int i = threadIdx.x; i < n; i += 256) dst[i] = piece.w[i];
}

// The device address of `scratch` on the current device, looked up once per device (the array's name is only a
// host-side handle, never a device address: host code uses the pointer returned here).
constexpr int MAX_DEVICES = 64;
int32_t static_scratch_ptr(void** out) {
    static std::mutex mu;
    static void* ptr[MAX_DEVICES] = {nullptr};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_err(e);
    if (dev < 0 || dev >= MAX_DEVICES) return GDN_ERR_COUNT;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_err(e);
        if (!p) return GDN_ERR_NULL;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return GDN_OK;
}

// ------------------------------------------------------------------ plan staging (pinned host memory)
// A ring of pinned buffers, each with the event of its last upload: a call waits (on the host) only when the
// ring has gone round and the upload that used its buffer PLAN_RING calls ago has not left it yet, so
// back-to-back short calls do not stall the host on one another.
constexpr int PLAN_RING = 8;
struct Staging {
    std::mutex mu;
    struct Slot {
        void* host = nullptr;
        size_t bytes = 0;
        hipEvent_t done = nullptr;
        bool pending = false;
    } slot[PLAN_RING];
    int next = 0;
};
Staging g_staging;

}  // namespace

// Copies `bytes` from `src` into pinned memory and enqueues its upload to `dst` (declared in gdn_host.h:
// the layer front end and the attention side upload their index arrays the same way).
int32_t upload_plan(const void* src, size_t bytes, void* dst, hipStream_t stream) {
    std::lock_guard<std::mutex> lock(g_staging.mu);
    Staging::Slot& s = g_staging.slot[g_staging.next];
    g_staging.next = (g_staging.next + 1) % PLAN_RING;
    if (!s.done) {
        const hipError_t e = hipEventCreateWithFlags(&s.done, hipEventDisableTiming);
        if (e != hipSuccess) return hip_err(e);
    }
    if (s.pending) {  // the upload that last used this buffer must have left it
        const hipError_t e = hipEventSynchronize(s.done);
        if (e != hipSuccess) return hip_err(e);
        s.pending = false;
    }
    if (s.bytes < bytes) {
        if (s.host) (void)hipHostFree(s.host);
        s.host = nullptr;
        s.bytes = 0;
        const size_t want = std::max<size_t>(bytes * 2, 1 << 16);
        const hipError_t e = hipHostMalloc(&s.host, want, hipHostMallocDefault);
        if (e != hipSuccess) return hip_err(e);
        s.bytes = want;
    }
    std::memcpy(s.host, src, bytes);
    hipError_t e = hipMemcpyAsync(dst, s.host, bytes, hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return hip_err(e);
    e = hipEventRecord(s.done, stream);
    if (e != hipSuccess) return hip_err(e);
    s.pending = true;
    return GDN_OK;
}

namespace {

// ------------------------------------------------------------------ optional per-kernel timing
// When switched on, the kernel launches of a prefill call are separated by events on the
// caller's stream (one before the first launch, one after each); collect() waits for them and
// sums the intervals per kernel kind.  Off by default: nothing is recorded.
struct Profiler {
    struct Mark { hipEvent_t ev; int kind; };   // kind of the launch that ENDS at ev; -1: a chain starts
    std::mutex mu;
    bool on = false;
    std::vector<hipEvent_t> spare;
    std::vector<Mark> marks;
    double ms[2] = {0.0, 0.0};   // 0: preparation, 1: recurrence
    int64_t launches[2] = {0, 0};
    int64_t calls = 0;

    hipEvent_t get() {
        if (!spare.empty()) {
            hipEvent_t e = spare.back();
            spare.pop_back();
            return e;
        }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
    void recycle() {
        for (auto& m : marks) spare.push_back(m.ev);
        marks.clear();
    }
};
Profiler g_prof;

// One call's chain of marks.
struct ProfChain {
    hipStream_t stream;
    bool on;
    explicit ProfChain(hipStream_t s) : stream(s) {
        std::lock_guard<std::mutex> lock(g_prof.mu);
        on = g_prof.on;
        if (on) mark_locked(-1);
    }
    void mark(int kind) {
        if (!on) return;
        std::lock_guard<std::mutex> lock(g_prof.mu);
        mark_locked(kind);
    }
private:
    void mark_locked(int kind) {
        hipEvent_t e = g_prof.get();
        if (!e) { on = false; return; }
        (void)hipEventRecord(e, stream);
        g_prof.marks.push_back({e, kind});
    }
};

// ------------------------------------------------------------------ host tier
int32_t check_tier_args(const void* host_pool, int64_t host_stride, int32_t host_n, const int32_t* host_ids,
                        const void* dev_pool, int64_t dev_stride, int32_t dev_n, const int32_t* dev_ids, int32_t n,
                        int64_t state_elems) {
    if (n < 0 || host_n < 0 || dev_n < 0 || state_elems < 0) return GDN_ERR_COUNT;
    if (n == 0 || state_elems == 0) return GDN_OK;
    if (!host_pool || !dev_pool || !host_ids || !dev_ids) return GDN_ERR_NULL;
    if (!aligned16(host_pool) || !aligned16(dev_pool)) return GDN_ERR_ALIGN;
    if ((state_elems & 3) || (host_stride & 3) || (dev_stride & 3)) return GDN_ERR_ALIGN;
    if (host_stride < state_elems || dev_stride < state_elems) return GDN_ERR_SHAPE;
    for (int32_t i = 0; i < n; ++i)
        if (host_ids[i] < 0 || host_ids[i] >= host_n || dev_ids[i] < 0 || dev_ids[i] >= dev_n) return GDN_ERR_SLOT_RANGE;
    return GDN_OK;
}

// Read-after-write hazards between the source and the destination slots of one call, by ADDRESS (the two pools may
// be the same memory under different base pointers or strides).  A request may store a state over its own start
// state when the two slots are the very same memory (the chain reads it before it writes); every other overlap of
// a destination with a source that is read in this call is an error: another workgroup may still be reading it.
int32_t check_slot_overlap(int32_t n_req, const float* src, int64_t src_stride, const int32_t* src_slot, const int32_t* emit_cu,
                           const float* dst, int64_t dst_stride, const int32_t* emit_slot, int64_t slot_elems) {
    if (!src || !dst || slot_elems <= 0) return GDN_OK;
    struct Range { uintptr_t lo, hi; int32_t req; };
    std::vector<Range> d;
    const uintptr_t bytes = (uintptr_t)slot_elems * sizeof(float);
    for (int32_t r = 0; r < n_req; ++r)
        for (int32_t e = emit_cu[r]; e < emit_cu[r + 1]; ++e) {
            const uintptr_t lo = reinterpret_cast<uintptr_t>(dst + (int64_t)emit_slot[e] * dst_stride);
            d.push_back({lo, lo + bytes, r});
        }
    if (d.empty()) return GDN_OK;
    std::sort(d.begin(), d.end(), [](const Range& a, const Range& b) { return a.lo < b.lo; });
    for (int32_t r = 0; r < n_req; ++r) {
        if (src_slot[r] < 0) continue;
        const uintptr_t lo = reinterpret_cast<uintptr_t>(src + (int64_t)src_slot[r] * src_stride), hi = lo + bytes;
        // destinations are disjoint and sorted: the candidates are the last one starting at or below lo and those after it
        auto it = std::upper_bound(d.begin(), d.end(), lo, [](uintptr_t x, const Range& a) { return x < a.lo; });
        if (it != d.begin()) --it;
        for (; it != d.end() && it->lo < hi; ++it) {
            if (it->hi <= lo) continue;
            if (it->req == r && it->lo == lo) continue;   // its own start state, the same memory exactly
            return GDN_ERR_SLOT_HAZARD;
        }
    }
    return GDN_OK;
}

// ------------------------------------------------------------------ kernel dispatch
template <typename E, int DK, int DV>
int64_t unit_bytes_of() { return UnitLayout<E, DK, DV>::UNIT_BYTES; }

int64_t unit_bytes(const gdn_shape& s) {
    if (s.in_dtype == GDN_F32) return unit_bytes_of<float, 64, 64>();
    return s.d_k == 64 ? unit_bytes_of<half_t, 64, 64>() : unit_bytes_of<half_t, 128, 128>();
}

// Compute units of the current device, looked up once (the variant choices below are sized by it).
int chip_cus() {
    static const int v = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
        return cus;
    }();
    return v;
}

template <typename E, int DK, int DV, int NW>
hipError_t launch_recur_nw(const RecurArgs& ra, int64_t n_chains, hipStream_t stream) {
    constexpr int SG = (DV / 32) / NW;
    constexpr int smem = recur_smem_bytes<E, DK, DV>();
    // once per process, also when several host threads make their first call together
    static std::once_flag once;
    static hipError_t once_err = hipSuccess;
    std::call_once(once, [] { once_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gdn_recur_kernel<E, DK, DV, NW>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, smem); });
    if (once_err != hipSuccess) return once_err;
    hipLaunchKernelGGL((gdn_recur_kernel<E, DK, DV, NW>), dim3((unsigned)(n_chains * SG)), dim3(64 * NW), smem, stream, ra);
    return hipGetLastError();
}

template <typename E, int DK, int DV, int NSW>
hipError_t launch_recur_ring(const RecurArgs& ra, int64_t n_chains, hipStream_t stream) {
    constexpr int smem = RingSmem<E, DK, DV, NSW>::BYTES;
    constexpr int SG = (DV / 32) / NSW;
    // once per process, also when several host threads make their first call together
    static std::once_flag once;
    static hipError_t once_err = hipSuccess;
    std::call_once(once, [] { once_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gdn_recur_ring_kernel<E, DK, DV, NSW>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, smem); });
    if (once_err != hipSuccess) return once_err;
    hipLaunchKernelGGL((gdn_recur_ring_kernel<E, DK, DV, NSW>), dim3((unsigned)(n_chains * SG)), dim3(64 * (NSW + 1)), smem, stream,
                       ra);
    return hipGetLastError();
}

template <typename E, int DK, int DV>
hipError_t launch_recur_quad(const RecurArgs& ra, int64_t n_chains, hipStream_t stream) {
    constexpr int smem = QuadSmem<E, DK, DV>::BYTES;
    // once per process, also when several host threads make their first call together
    static std::once_flag once;
    static hipError_t once_err = hipSuccess;
    std::call_once(once, [] { once_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gdn_recur_quad_kernel<E, DK, DV>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, smem); });
    if (once_err != hipSuccess) return once_err;
    hipLaunchKernelGGL((gdn_recur_quad_kernel<E, DK, DV>), dim3((unsigned)(n_chains * (DV / 32))), dim3(256), smem, stream, ra);
    return hipGetLastError();
}

// Latency variant with several slabs: the recurrence over slab s and the preparation of slab s+1
// are independent, so they share one launch, the recurrence workgroups first (they are
// dispatched first and each takes a whole compute unit), the preparation workgroups on the
// compute units that are left.  No synchronisation between the two roles: the dependences
// (slab s prepared before its recurrence, states carried from slab to slab) run from launch to
// launch.
template <typename E, int DK, int DV>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) gdn_quad_overlap_kernel(RecurArgs ra, PrepArgs pa,
                                                                                                         int n_recur) {
    if ((int)blockIdx.x < n_recur) recur_quad_body<E, DK, DV>(ra, (int)blockIdx.x, n_recur);
    else prep_body<E, DK, DV>(pa, (int)blockIdx.x - n_recur, (int)gridDim.x - n_recur);
}

template <typename E, int DK, int DV>
hipError_t launch_quad_overlap(const RecurArgs& ra, const PrepArgs& pa, int64_t n_chains, int64_t prep_items, int cus,
                               hipStream_t stream) {
    constexpr int smem = QuadSmem<E, DK, DV>::BYTES > PrepSmem<E, DK, DV>::BYTES ? QuadSmem<E, DK, DV>::BYTES
                                                                               : PrepSmem<E, DK, DV>::BYTES;
    // once per process, also when several host threads make their first call together
    static std::once_flag once;
    static hipError_t once_err = hipSuccess;
    std::call_once(once, [] { once_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&gdn_quad_overlap_kernel<E, DK, DV>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, smem); });
    if (once_err != hipSuccess) return once_err;
    const int n_recur = (int)(n_chains * (DV / 32));
    const int n_prep = (int)std::min<int64_t>(prep_items, std::max(cus - n_recur, 16));   // one workgroup per compute unit
    hipLaunchKernelGGL((gdn_quad_overlap_kernel<E, DK, DV>), dim3((unsigned)(n_recur + n_prep)), dim3(256), smem, stream, ra, pa,
                       n_recur);
    return hipGetLastError();
}

// Fused throughput kernel (bf16 inputs, d_k = d_v = 64 or 128): see gdn_fused_kernel.h.
// per_cu: workgroups that may share a compute unit (0 or more than fit: as many as fit).  Fewer than fit are enforced by asking
// for so much LDS per workgroup that one more would not fit; the grid is the compute units times that number.
constexpr int CU_LDS_BYTES = 160 * 1024;
template <bool O_BF16, int D, int GV>
hipError_t launch_fused_t(const FusedArgs& fa, int per_cu, hipStream_t stream) {
    typedef FusedSmem<D, GV> SM;
    static std::once_flag once;
    static hipError_t once_err = hipSuccess;
    static int cus = 1, fit = 1;
    std::call_once(once, [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gdn_fused_kernel<O_BF16, D, GV>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, CU_LDS_BYTES);
        int dev = 0, n_cu = 0, n_fit = 0;
        if (e == hipSuccess) e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n_fit, gdn_fused_kernel<O_BF16, D, GV>, 256 * GV, SM::BYTES);
        once_err = e;
        if (e == hipSuccess) { cus = std::max(1, n_cu); fit = std::max(1, n_fit); }
    });
    if (once_err != hipSuccess) return once_err;
    int lds = SM::BYTES, n = fit;
    if (per_cu >= 1 && per_cu < fit) {
        n = per_cu;
        lds = std::max(lds, (CU_LDS_BYTES / (per_cu + 1) + 256) & ~255);    // per_cu + 1 of these exceed a compute unit's LDS
    }
    hipLaunchKernelGGL((gdn_fused_kernel<O_BF16, D, GV>), dim3((unsigned)std::min<int64_t>(fa.n_chains, (int64_t)cus * n)), dim3(256 * GV),
                       lds, stream, fa);
    return hipGetLastError();
}
// gv = value heads per workgroup (1, or 2 when the heads of a pair share a query/key head); fa.n_chains counts groups of gv heads.
hipError_t launch_fused(const FusedArgs& fa, int d, int gv, int per_cu, hipStream_t stream) {
    if (gv == 2) {
        if (d == 64) return fa.o_bf16 ? launch_fused_t<true, 64, 2>(fa, per_cu, stream) : launch_fused_t<false, 64, 2>(fa, per_cu, stream);
        return fa.o_bf16 ? launch_fused_t<true, 128, 2>(fa, per_cu, stream) : launch_fused_t<false, 128, 2>(fa, per_cu, stream);
    }
    if (d == 64) return fa.o_bf16 ? launch_fused_t<true, 64, 1>(fa, per_cu, stream) : launch_fused_t<false, 64, 1>(fa, per_cu, stream);
    return fa.o_bf16 ? launch_fused_t<true, 128, 1>(fa, per_cu, stream) : launch_fused_t<false, 128, 1>(fa, per_cu, stream);
}

// How many fused workgroups share a compute unit (0: as many as fit).  A chunk of a chain takes less time when its
// workgroup has the compute unit to itself (measured at d = 128: 5.5 us against 6.8 us with two), so a call bound by its
// longest chain rather than by its volume runs better on fewer, faster workgroups.  Estimates: one per compute unit
// max(longest chain x 5.5 us, units x 0.0257 us) (all 256 busy, a chunk takes 6.6 us), two max(longest chain x 6.8 us,
// units x 0.0183 us).  Measured, one against two: 1024 chains of up to 66 chunks, 14.8 k units 0.431 against 0.449 ms; 384
// chains of up to 128 chunks, 28 k units 0.72 against 0.79; 512 chains, 39 k units 0.92 against 0.87; 1024 chains of up to 345
// chunks, 99.5 k units 2.56 against 2.31.  gdn_tune_fused_per_cu forces the number.
std::atomic<int32_t> g_forced_per_cu{-1};
inline int fused_wgs_per_cu(const gdn_shape& s, int gv, int64_t total_units, int32_t longest_chain_chunks) {
    const int forced = g_forced_per_cu.load();
    if (forced >= 1) return forced;
    if (s.d_k != 128 || gv != 1) return 0;
    const double cus = (double)chip_cus(), units = (double)total_units, longest = (double)longest_chain_chunks;   // (figures from 256 compute units)
    const double t1 = std::max(longest * 5.5, units * 0.0257 * 256.0 / cus);
    const double t2 = std::max(longest * 6.8, units * 0.0183 * 256.0 / cus);
    return t1 < t2 ? 1 : 0;
}

// Grouped value heads (H_v a multiple of H_qk): two value heads of one query/key head can share a workgroup of eight waves,
// which then reads and stages that head's q and k rows once for both (a fifth of a call's bytes with fp32 outputs).  It
// needs an even group size.  The eight waves move in step, where two workgroups of four on a compute unit overlap each
// other's phases, so a chunk of a chain takes longer (8.2 against 7.7 us at d = 128) and only calls bound by their
// volume gain.  Measured at d = 128, 8 query/key heads under 16 value heads, pairs against single heads: 32768 chains of
// up to 126 chunks 16.3 against 18.2 ms; 8192 chains 4.25 against 4.74; 4096 chains 2.29 against 2.32; 2048 chains 1.36
// either way; 2048 chains of up to 32 chunks 0.47 against 0.44; 1024 chains of up to 320 chunks 2.66 against 2.50.  At
// d = 64 a pair's 81 KB of LDS leave a compute unit one workgroup where three single-head ones fit, and pairs never won
// (9.47 against 9.56 ms on 32768 chains, 1.39 against 1.17 on 4096): forced only.  (Since then the one-head kernel has gained
// about 10 % and the pair kernel 5 % from changes to their loads and to the order of the chains: on the first of these calls
// 16.7 against 17.4 ms; the threshold was raised accordingly, pairs from three times the longest chain's time in volume.)  gdn_tune_fused_pair forces the choice.
std::atomic<int32_t> g_forced_pair{-1};
inline int fused_heads_per_wg(const gdn_shape& s, int64_t total_units, int32_t longest_chain_chunks) {
    if (s.H_qk <= 0 || s.H_v % s.H_qk != 0 || (s.H_v / s.H_qk) % 2 != 0) return 1;
    const int forced = g_forced_pair.load();
    if (forced >= 0) return forced != 0 ? 2 : 1;
    if (s.d_k != 128) return 1;
    return 0.0197 * (double)total_units >= 3.0 * 8.2 * (double)longest_chain_chunks ? 2 : 1;
}

// The fused kernel serialises a chain's preparation along the chain; it pays when chains are
// plentiful and the longest chain does not outlast the whole two-kernel run.  Estimates from
// figures measured on MI355X (bf16; one call of 4 to 64 requests of up to 8192 tokens, 16 heads,
// and the large configurations).  d = 128: fused, per chunk of one chain 5.5 us with one workgroup
// per compute unit (up to 256 chains) and 6.8 us with two, per (chunk, chain) unit of a large call
// 0.0183 us; two-kernel path 0.056 us per unit plus about 0.15 ms.  Measured, fused against
// two-kernel: 64 chains 0.60 against 0.40 ms, 96 chains 0.61 against 0.52, 128 chains 0.62 against
// 0.63, 160 chains 0.70 against 0.85, 256 chains 0.70 against 1.14, 512 chains 0.87 against 2.04,
// 1024 chains 1.49 against 4.17.  d = 64: 3.4 / 4.4 us per chunk, 0.0094 us per unit; two-kernel
// path 0.036 us per unit plus about 0.1 ms (requests of up to 4096 tokens: 96 chains 0.21 against
// 0.17 ms, 128 chains 0.21 against 0.22, 256 chains 0.25 against 0.39, 1024 chains 0.45 against
// 1.48).  gdn_tune_fused forces the choice.
std::atomic<int32_t> g_forced_fused{-1};
inline bool fused_applies(const gdn_shape& s) { return s.in_dtype == GDN_BF16 && s.d_k == s.d_v && (s.d_k == 128 || s.d_k == 64); }
inline bool choose_fused(const gdn_shape& s, int64_t n_chains, int64_t total_units, int32_t longest_chain_chunks) {
    if (!fused_applies(s)) return false;
    const int forced = g_forced_fused.load();
    if (forced >= 0) return forced != 0;
    if (n_chains < 128) return false;
    const bool big = s.d_k == 128;
    const double per_chunk = n_chains <= chip_cus() ? (big ? 5.5 : 3.4) : (big ? 6.8 : 4.4);   // us: one or two workgroups per compute unit
    const double t_two = (big ? 0.056 : 0.036) * (double)total_units + (big ? 150.0 : 100.0);
    const double t_fused = std::max((big ? 0.0183 : 0.0094) * (double)total_units, per_chunk * (double)longest_chain_chunks);
    return t_fused < t_two;
}

// Which recurrence variant a call gets: 1 = latency variant (few chains), else the number of
// d_v slices (waves) per workgroup of the throughput variant.
inline int pick_waves(int64_t n_chains, int ns, bool frag16) {
    int nw = ns;
    while (nw > 1 && n_chains * (ns / nw) < 512) nw >>= 1;
    // A latency-variant workgroup fills a compute unit's LDS: with more of them than compute units
    // they would run in turns (measured: 96 chains 1.0 ms against 0.70 ms with two slices per
    // workgroup).
    if (nw == 1 && n_chains * ns > chip_cus()) nw = 2;
    if (nw == 1 && !frag16) nw = 2;   // fp32 operands: the latency variant's registers are sized for 16-byte fragments
    return nw;
}

// Latency variant: does the preparation of the next slab share the recurrence's launch?  Only while the
// recurrence leaves half of the compute units to it: the two kinds of workgroup cannot share a compute
// unit's LDS, so beyond that the preparation would be left with a few workgroups (measured at 64 chains:
// 1.77 ms shared, 0.56 ms apart).
inline bool latency_shared(int64_t n_chains, int ns) {
    return n_chains * ns <= chip_cus() / 2;
}

// Chunk rounds per slab.  In the latency variant the slab should stay cache resident between the preparation launch
// that writes it and the recurrence launch that reads it back (budget), and a preparation
// launch should fill the chip a whole number of times (512 = two of its workgroups on each of
// the 256 compute units); the throughput variants only bound the workspace.  gdn_tune_slab_rounds
// overrides the choice.
std::atomic<int32_t> g_forced_rounds{0};
inline int32_t slab_rounds(int64_t n_chains, int64_t unit_bytes, int nw, int ns) {
    const int32_t forced = g_forced_rounds.load();
    if (forced > 0) return forced;
    // Latency variant with launches apart (33 to 64 chains at four slices): every slab costs two launches
    // and a hand-over of the states, so slabs are long (measured at 64 chains: 0.56 ms with 8 rounds, 0.31 ms
    // with 64).
    if (nw == 1 && !latency_shared(n_chains, ns)) return 64;
    // Throughput variants: the states are carried through memory from slab to slab (d_v d_k floats per
    // chain each way), so slabs are as long as the byte budget allows.
    const int64_t budget = nw == 1 ? (int64_t)48 << 20 : (int64_t)1 << 30;
    int64_t r = std::max<int64_t>(1, budget / std::max<int64_t>(1, n_chains * unit_bytes));
    const int64_t q = std::max<int64_t>(1, 512 / std::max<int64_t>(1, n_chains));
    r = std::max(q, r / q * q);
    return (int32_t)std::min<int64_t>(r, 1 << 16);
}

template <typename E, int DK, int DV>
int32_t launch_all(const gdn_shape& s, PrepArgs pa, RecurArgs ra, int32_t n_req, int32_t max_chunks_per_req,
                   char* slab_base, int64_t slab_bytes, int32_t n_bufs, hipStream_t stream) {
    typedef PrepSmem<E, DK, DV> SM;
    // workgroups of the preparation kernel the chip holds at once (per kernel instance)
    static std::once_flag once;
    static hipError_t once_err = hipSuccess;
    static int prep_slots = 1;
    std::call_once(once, [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gdn_prep_kernel<E, DK, DV>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, SM::BYTES);
        int dev = 0, cus = 0, per_cu = 0;
        if (e == hipSuccess) e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess)
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gdn_prep_kernel<E, DK, DV>, 256, SM::BYTES);
        once_err = e;
        if (e == hipSuccess) prep_slots = std::max(1, cus * per_cu);
    });
    if (once_err != hipSuccess) return hip_err(once_err);
    const int units = s.L * s.H_v;
    const int64_t n_chains = (int64_t)n_req * units;
    constexpr int NS = DV / 32;
    const int nw = pick_waves(n_chains, NS, sizeof(typename Elem<E>::Frag) == 16);
    const int32_t R = pa.R;
    const int32_t n_slabs = (max_chunks_per_req + R - 1) / R;

    // Slab after slab on the caller's stream: the units one preparation launch writes are read
    // back by the recurrence launch right behind it while they are still in the caches.  With two
    // slab buffers (latency variant) the preparation of the next slab shares the recurrence's launch.
    ProfChain prof(stream);
    const bool overlap = nw == 1 && n_bufs >= 2 && n_slabs > 1 && sizeof(typename Elem<E>::Frag) == 16 && latency_shared(n_chains, NS);
    const int64_t items = (int64_t)n_req * R * units;
    if (items > INT32_MAX) return GDN_ERR_COUNT;
    auto launch_prep = [&](int32_t sb, char* buf, bool with_copies) -> hipError_t {
        PrepArgs pl = pa;
        pl.ws_units = buf;
        pl.slab_begin = sb * R;
        if (!with_copies) pl.n_copy_wgs = 0;   // the start states travel with the first launch only
        hipLaunchKernelGGL((gdn_prep_kernel<E, DK, DV>),
                           dim3((unsigned)(std::min<int64_t>(items, prep_slots) + pl.n_copy_wgs)), dim3(256), SM::BYTES, stream, pl);
        return hipGetLastError();
    };
    for (int32_t sb = 0; sb < n_slabs; ++sb) {
        char* buf = slab_base + (overlap ? (sb & 1) * slab_bytes : 0);
        hipError_t e = hipSuccess;
        if (!overlap || sb == 0) {
            e = launch_prep(sb, buf, sb == 0);
            if (e != hipSuccess) return hip_err(e);
            prof.mark(0);
        }
        ra.ws_units = buf;
        ra.slab_begin = sb * R;
        // Recurrence variant: with enough chains to fill the chip, NS slices (waves) of a chain
        // share one workgroup and one LDS copy of the chunk operands; with fewer, two slices per
        // workgroup; with too few to occupy every compute unit, the latency variant.
        if constexpr (sizeof(typename Elem<E>::Frag) == 16) {
            if (nw == 1) {
                if (overlap && sb + 1 < n_slabs) {
                    PrepArgs pl = pa;
                    pl.ws_units = slab_base + ((sb + 1) & 1) * slab_bytes;
                    pl.slab_begin = (sb + 1) * R;
                    pl.n_copy_wgs = 0;
                    e = launch_quad_overlap<E, DK, DV>(ra, pl, n_chains, items, chip_cus(), stream);
                } else {
                    e = launch_recur_quad<E, DK, DV>(ra, n_chains, stream);
                }
            }
        }
        // Throughput variants.  While two slices per workgroup still give at most one workgroup per compute
        // unit (65 to 128 chains at four slices), the ring variant: no register staging, the next chunk lands
        // in LDS while this one is worked on (measured: 96 chains 0.51 against 0.58 ms, 128 chains 0.57 against
        // 0.64 ms).
        bool ring = false;
        if constexpr (sizeof(typename Elem<E>::Frag) == 16 && NS == 4) {
            if (nw >= 2 && n_chains * 2 <= chip_cus()) {
                e = launch_recur_ring<E, DK, DV, 2>(ra, n_chains, stream);
                ring = true;
            }
        }
        if (!ring && nw == 2) e = launch_recur_nw<E, DK, DV, 2>(ra, n_chains, stream);
        else if (!ring && nw > 2) e = launch_recur_nw<E, DK, DV, NS>(ra, n_chains, stream);
        if (e != hipSuccess) return hip_err(e);
        prof.mark(1);
    }
    {
        std::lock_guard<std::mutex> lock(g_prof.mu);
        if (g_prof.on) g_prof.calls += 1;
    }
    return GDN_OK;
}

}  // namespace
}  // namespace gdn

using namespace gdn;

extern "C" {

int32_t gdn_version(void) { return 100; }

#ifdef GDN_PHASE_STAMPS
// Profiling build only: the cycle stamps the fused kernel left (64 workgroups x 4 waves x 16 stamps), after a device
// synchronisation.  Not declared in the public header: the product library does not export it.
extern "C" int32_t gdn_phase_stamps(unsigned long long* out) {
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpyFromSymbol(out, HIP_SYMBOL(gdn::g_phase_ts), sizeof(unsigned long long) * 64 * 4 * 16);
    return e == hipSuccess ? GDN_OK : GDN_ERR_HIP - (int32_t)e;
}
#endif

int32_t gdn_tune_fused(int32_t mode) {
    return g_forced_fused.exchange(mode < 0 ? -1 : (mode != 0));
}

int32_t gdn_tune_fused_per_cu(int32_t n) {
    return g_forced_per_cu.exchange(n >= 1 ? n : -1);
}

int32_t gdn_tune_fused_pair(int32_t mode) {
    return g_forced_pair.exchange(mode < 0 ? -1 : (mode != 0));
}

int32_t gdn_tune_slab_rounds(int32_t rounds) {
    return g_forced_rounds.exchange(rounds > 0 ? rounds : 0);
}

int32_t gdn_profile_enable(int32_t on) {
    std::lock_guard<std::mutex> lock(g_prof.mu);
    g_prof.on = on != 0;
    if (on) {
        g_prof.recycle();
        g_prof.ms[0] = g_prof.ms[1] = 0.0;
        g_prof.launches[0] = g_prof.launches[1] = 0;
        g_prof.calls = 0;
    }
    return GDN_OK;
}

int32_t gdn_profile_collect(double* prep_ms, double* recur_ms, int64_t* calls, int64_t* prep_launches,
                            int64_t* recur_launches) {
    std::lock_guard<std::mutex> lock(g_prof.mu);
    for (size_t i = 0; i < g_prof.marks.size(); ++i) {
        const Profiler::Mark& m = g_prof.marks[i];
        if (m.kind < 0) continue;
        hipError_t e = hipEventSynchronize(m.ev);
        if (e != hipSuccess) return hip_err(e);
        float t = 0.f;
        e = hipEventElapsedTime(&t, g_prof.marks[i - 1].ev, m.ev);
        if (e != hipSuccess) return hip_err(e);
        g_prof.ms[m.kind] += t;
        g_prof.launches[m.kind] += 1;
    }
    g_prof.recycle();
    if (prep_ms) *prep_ms = g_prof.ms[0];
    if (recur_ms) *recur_ms = g_prof.ms[1];
    if (calls) *calls = g_prof.calls;
    if (prep_launches) *prep_launches = g_prof.launches[0];
    if (recur_launches) *recur_launches = g_prof.launches[1];
    return GDN_OK;
}

int32_t gdn_probe_ceilings(void* scratch, int64_t scratch_bytes, double* mfma_f16_tflops, double* copy_gbs,
                           void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    if (!scratch) return GDN_ERR_NULL;
    if (!aligned16(scratch)) return GDN_ERR_ALIGN;
    if (scratch_bytes < (1 << 20)) return GDN_ERR_WORKSPACE;
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_err(e);
    const int blocks = std::max(1, cus) * 2;   // two workgroups of four waves per compute unit
    if (scratch_bytes < (int64_t)blocks * PROBE_THREADS * (int64_t)sizeof(float)) return GDN_ERR_WORKSPACE;
    hipEvent_t ev[2] = {nullptr, nullptr};
    for (auto& x : ev)
        if ((e = hipEventCreate(&x)) != hipSuccess) return hip_err(e);
    auto timed = [&](auto&& launch, int reps, double* ms) -> hipError_t {
        launch();   // warm-up
        hipError_t r = hipEventRecord(ev[0], stream);
        if (r != hipSuccess) return r;
        for (int i = 0; i < reps; ++i) launch();
        if ((r = hipGetLastError()) != hipSuccess) return r;
        if ((r = hipEventRecord(ev[1], stream)) != hipSuccess) return r;
        if ((r = hipEventSynchronize(ev[1])) != hipSuccess) return r;
        float t = 0.f;
        r = hipEventElapsedTime(&t, ev[0], ev[1]);
        *ms = (double)t / reps;
        return r;
    };
    double ms = 0.0;
    const int iters = 4096;
    e = timed([&] { hipLaunchKernelGGL(probe_mfma_kernel, dim3(blocks), dim3(PROBE_THREADS), 0, stream,
                                       reinterpret_cast<float*>(scratch), iters); }, 3, &ms);
    if (e == hipSuccess && mfma_f16_tflops) {
        const double flop = (double)blocks * (PROBE_THREADS / 64) * iters * PROBE_MFMA_PER_ITER * (2.0 * 32 * 32 * 16);
        *mfma_f16_tflops = flop / (ms * 1e-3) / 1e12;
    }
    if (e == hipSuccess) {
        const int64_t half = scratch_bytes / 2 / 16 * 16;
        const f32x4* src = reinterpret_cast<const f32x4*>(scratch);
        f32x4* dst = reinterpret_cast<f32x4*>(reinterpret_cast<char*>(scratch) + half);
        const int64_t n4 = half / 16;
        e = timed([&] { hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)((n4 + PROBE_THREADS - 1) / PROBE_THREADS)), dim3(PROBE_THREADS), 0,
                                           stream, src, dst, n4); },
                  5, &ms);
        if (e == hipSuccess && copy_gbs) *copy_gbs = 2.0 * (double)half / (ms * 1e-3) / 1e9;
    }
    for (auto& x : ev) (void)hipEventDestroy(x);
    return e == hipSuccess ? GDN_OK : hip_err(e);
}

int32_t gdn_deepest_ckpt(const int32_t* pos, int32_t M, int32_t t) {
    if (!pos || M <= 0) return -1;
    // largest i with pos[i] <= t (pos strictly increasing)
    const int32_t* it = std::upper_bound(pos, pos + M, t);
    return (int32_t)(it - pos) - 1;
}

int32_t gdn_plan_chunks(int32_t n_req, const int32_t* cu_seqlens, const int32_t* start_pos, const int32_t* emit_cu,
                        const int32_t* emit_pos, int32_t* chunk_tok0, int32_t* chunk_len, int32_t* chunk_emit,
                        int32_t* req_chunk_cu, int32_t capacity) {
    ChunkPlan plan;
    const int32_t rc = plan_chunks(n_req, cu_seqlens, start_pos, emit_cu, emit_pos, &plan);
    if (rc != GDN_OK) return rc;
    const int32_t nc = (int32_t)plan.chunk_tok0.size();
    if (nc > capacity) return GDN_ERR_WORKSPACE;
    if (nc > 0 && (!chunk_tok0 || !chunk_len || !chunk_emit)) return GDN_ERR_NULL;
    if (!req_chunk_cu) return GDN_ERR_NULL;
    if (nc > 0) {
        std::memcpy(chunk_tok0, plan.chunk_tok0.data(), sizeof(int32_t) * nc);
        std::memcpy(chunk_len, plan.chunk_len.data(), sizeof(int32_t) * nc);
        std::memcpy(chunk_emit, plan.chunk_emit.data(), sizeof(int32_t) * nc);
    }
    std::memcpy(req_chunk_cu, plan.req_chunk_cu.data(), sizeof(int32_t) * (n_req + 1));
    return nc;
}

static int64_t plan_bytes(int64_t n_chunks, int64_t n_req) {
    return align_up((3 * n_chunks + 4 * n_req + 2) * (int64_t)sizeof(int32_t), 256);
}

// Workspace = [plan | carried states | slab buffers].  A slab buffer holds the units of R chunk
// rounds of every chain; slabs are processed one after the other.  The throughput variants
// reuse one buffer; the latency variant alternates between two, so that the next slab can be
// prepared while the current one is consumed.
struct WsLayout {
    int32_t R, n_bufs;
    int64_t plan, carry, slab, total;
};
// n_chunks: chunks of the whole call; max_rounds: chunks of its longest request (or a bound)
static WsLayout ws_layout(const gdn_shape& s, int64_t n_chunks, int64_t max_rounds, int32_t n_req) {
    const int64_t units = (int64_t)s.L * s.H_v, n_chains = units * n_req, ub = unit_bytes(s);
    const int nw = pick_waves(n_chains, s.d_v / 32, s.in_dtype != GDN_F32);
    WsLayout w;
    w.R = (int32_t)std::max<int64_t>(1, std::min<int64_t>(slab_rounds(n_chains, ub, nw, s.d_v / 32), max_rounds));
    w.plan = plan_bytes(n_chunks, n_req);
    w.carry = align_up(n_chains * s.d_v * s.d_k * (int64_t)sizeof(float), 256);
    w.slab = n_chains * w.R * ub;
    w.n_bufs = (nw == 1 && latency_shared(n_chains, s.d_v / 32)) ? 2 : 1;   // two buffers: the next slab is prepared while this one is consumed
    w.total = w.plan + w.carry + w.n_bufs * w.slab;
    return w;
}

int64_t gdn_workspace_bytes(const gdn_shape* shape, int32_t n_req, int64_t total_tokens, int32_t n_emit) {
    const int32_t rc = check_shape(shape);
    if (rc != GDN_OK) return rc;
    if (n_req < 0 || total_tokens < 0 || n_emit < 0) return GDN_ERR_COUNT;
    const int64_t max_chunks = total_tokens / GDN_CHUNK + n_req + n_emit + 1;
    return ws_layout(*shape, max_chunks, max_chunks, n_req).total;
}

int64_t gdn_workspace_bytes_fused(const gdn_shape* shape, int32_t n_req, int64_t total_tokens, int32_t n_emit) {
    const int32_t rc = check_shape(shape);
    if (rc != GDN_OK) return rc;
    if (n_req < 0 || total_tokens < 0 || n_emit < 0) return GDN_ERR_COUNT;
    if (!fused_applies(*shape)) return gdn_workspace_bytes(shape, n_req, total_tokens, n_emit);
    return plan_bytes(total_tokens / GDN_CHUNK + n_req + n_emit + 1, n_req);
}

int32_t ckpt_gather(const float* pool, int64_t slot_stride, int32_t n_slots, const int32_t* slot_ids, int32_t n,
                    float* dst, int64_t dst_stride, int64_t state_elems, void* stream) {
    const int32_t rc = check_copy_args(pool, slot_stride, n_slots, slot_ids, n, dst, dst_stride, state_elems, true);
    if (rc != GDN_OK || n == 0 || state_elems == 0) return rc;
    return launch_copy<true>(pool, dst, slot_stride, dst_stride, state_elems, slot_ids, n, (hipStream_t)stream);
}

int32_t ckpt_scatter(float* pool, int64_t slot_stride, int32_t n_slots, const int32_t* slot_ids, int32_t n,
                     const float* src, int64_t src_stride, int64_t state_elems, void* stream) {
    const int32_t rc = check_copy_args(pool, slot_stride, n_slots, slot_ids, n, src, src_stride, state_elems, false);
    if (rc != GDN_OK || n == 0 || state_elems == 0) return rc;
    std::vector<int32_t> sorted(slot_ids, slot_ids + n);
    std::sort(sorted.begin(), sorted.end());
    if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return GDN_ERR_SLOT_DUP;
    return launch_copy<false>(src, pool, src_stride, slot_stride, state_elems, slot_ids, n, (hipStream_t)stream);
}

// The body of gdn_resume_prefill; with POOL_HOST the start states live in a pinned host pool
// and are first copied to a staging area behind the workspace proper; with POOL_DEVICE_STATIC the
// plan image goes to the library's static array and the fused kernel runs.
enum PoolKind { POOL_DEVICE = 0, POOL_HOST = 1, POOL_DEVICE_STATIC = 2 };
static int32_t prefill_impl(const gdn_shape* shape, const void* q, const void* k, const void* v, const void* beta,
                            const void* gate, int32_t n_req, const int32_t* cu_seqlens, const int32_t* start_pos,
                            const float* state_src, int64_t src_slot_stride, int32_t src_n_slots,
                            const int32_t* src_slot, const int32_t* emit_cu, const int32_t* emit_pos,
                            float* state_dst, int64_t dst_slot_stride, int32_t dst_n_slots, const int32_t* emit_slot,
                            void* o, void* workspace, int64_t workspace_bytes, void* stream_v, PoolKind kind) {
    hipStream_t stream = (hipStream_t)stream_v;
    int32_t rc = check_shape(shape);
    if (rc != GDN_OK) return rc;
    const gdn_shape& s = *shape;
    const bool src_on_host = kind == POOL_HOST;
    const bool no_alloc = kind == POOL_DEVICE_STATIC;   // plan image in the library's static array, written by kernel arguments
    if (no_alloc) {
        if (!fused_applies(s)) return GDN_ERR_SHAPE;
        rc = static_scratch_ptr(&workspace);
        if (rc != GDN_OK) return rc;
        workspace_bytes = STATIC_SCRATCH_BYTES;
    }

    ChunkPlan plan;
    rc = plan_chunks(n_req, cu_seqlens, start_pos, emit_cu, emit_pos, &plan);
    if (rc != GDN_OK) return rc;
    const int64_t total_tokens = cu_seqlens[n_req];
    if (total_tokens > s.T_alloc) return GDN_ERR_SEQLENS;
    const int32_t n_emit = emit_cu[n_req];
    rc = check_slots(n_req, src_slot, src_n_slots, emit_cu, emit_slot, dst_n_slots);
    if (rc != GDN_OK) return rc;

    const int64_t slot_elems = (int64_t)s.L * s.H_v * s.d_v * s.d_k;
    bool any_src = false;
    for (int32_t r = 0; r < n_req; ++r) any_src |= src_slot[r] >= 0;
    if (any_src) {
        if (!state_src) return GDN_ERR_NULL;
        if (!aligned16(state_src) || (src_slot_stride & 3)) return GDN_ERR_ALIGN;
        if (src_slot_stride < slot_elems) return GDN_ERR_SHAPE;
    }
    if (n_emit > 0) {
        if (!state_dst) return GDN_ERR_NULL;
        if (!aligned16(state_dst) || (dst_slot_stride & 3)) return GDN_ERR_ALIGN;
        if (dst_slot_stride < slot_elems) return GDN_ERR_SHAPE;
    }
    if (!src_on_host) {
        rc = check_slot_overlap(n_req, state_src, src_slot_stride, src_slot, emit_cu, state_dst, dst_slot_stride, emit_slot,
                                slot_elems);
        if (rc != GDN_OK) return rc;
    }
    const int32_t n_chunks = (int32_t)plan.chunk_tok0.size();
    if (n_chunks == 0) return GDN_OK;  // nothing to replay
    if (!q || !k || !v || !beta || !gate || !o) return GDN_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return GDN_ERR_ALIGN;

    // The fused kernel needs the plan image only; the two-kernel path needs the carried states and a slab as well.
    // A workspace too small for the two-kernel path but large enough for the fused kernel gets the fused kernel
    // whatever the estimate says (gdn_workspace_bytes_fused is the size that asks for this).
    WsLayout wl = ws_layout(s, n_chunks, plan.max_chunks_per_req, n_req);
    int32_t n_staged = 0;
    if (src_on_host)
        for (int32_t r = 0; r < n_req; ++r) n_staged += src_slot[r] >= 0;
    const int64_t staged_bytes = src_on_host ? (int64_t)n_staged * slot_elems * (int64_t)sizeof(float) : 0;
    bool use_fused = choose_fused(s, (int64_t)n_req * s.L * s.H_v, (int64_t)n_chunks * s.L * s.H_v, plan.max_chunks_per_req);
    if (!use_fused && fused_applies(s) && g_forced_fused.load() != 0 &&
        workspace_bytes < align_up(wl.total, 256) + staged_bytes)
        use_fused = true;
    if (no_alloc) {
        if (wl.plan > STATIC_SCRATCH_BYTES) return GDN_ERR_STATIC_LIMIT;
        use_fused = true;
    }
    if (use_fused) {
        wl.carry = 0;
        wl.slab = 0;
        wl.n_bufs = 0;
        wl.total = wl.plan;
    }
    const int64_t staging_off = align_up(wl.total, 256);
    const int64_t need = src_on_host ? staging_off + staged_bytes : wl.total;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return GDN_ERR_WORKSPACE;
    if (workspace_bytes < need) return GDN_ERR_WORKSPACE;

    // ---- plan image: [tok0 | len | emit slot] per chunk, [chunk_cu | src slot | order | staged host slots] per request, and
    //      one word that starts at zero: the fused kernel's counter of chains handed out
    std::vector<int32_t> img((size_t)(3 * (int64_t)n_chunks + 4 * (int64_t)n_req + 2));
    int32_t* p_tok0 = img.data();
    int32_t* p_len = p_tok0 + n_chunks;
    int32_t* p_eslot = p_len + n_chunks;
    int32_t* p_cu = p_eslot + n_chunks;
    int32_t* p_src = p_cu + (n_req + 1);
    int32_t* p_order = p_src + n_req;
    for (int32_t c = 0; c < n_chunks; ++c) {
        p_tok0[c] = plan.chunk_tok0[c];
        p_len[c] = plan.chunk_len[c];
        p_eslot[c] = plan.chunk_emit[c] >= 0 ? emit_slot[plan.chunk_emit[c]] : -1;
    }
    std::memcpy(p_cu, plan.req_chunk_cu.data(), sizeof(int32_t) * (n_req + 1));
    std::memcpy(p_src, src_slot, sizeof(int32_t) * n_req);
    if (src_on_host) {   // the recurrence reads request r's start state from its place in the staging area
        int32_t* p_staged = p_order + n_req;
        int32_t at = 0;
        for (int32_t r = 0; r < n_req; ++r) {
            if (src_slot[r] >= 0) p_staged[at] = src_slot[r];
            p_src[r] = src_slot[r] >= 0 ? at++ : -1;
        }
    }
    const std::vector<int32_t> order = longest_first(plan, n_req);
    std::memcpy(p_order, order.data(), sizeof(int32_t) * n_req);

    if (no_alloc) {
        // by value in the arguments of a few small launches: no staging buffer, nothing for a replay to find changed
        for (size_t at = 0; at < img.size(); at += PLAN_PIECE_WORDS) {
            PlanPiece piece;
            const int32_t n = (int32_t)std::min<size_t>(PLAN_PIECE_WORDS, img.size() - at);
            std::memcpy(piece.w, img.data() + at, sizeof(int32_t) * (size_t)n);
            hipLaunchKernelGGL(plan_write_kernel, dim3(1), dim3(256), 0, stream, piece, reinterpret_cast<int32_t*>(workspace) + at, n);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return hip_err(e);
        }
    } else {
        rc = upload_plan(img.data(), img.size() * sizeof(int32_t), workspace, stream);
        if (rc != GDN_OK) return rc;
    }

    const int32_t* d = reinterpret_cast<const int32_t*>(workspace);
    char* slab_base = reinterpret_cast<char*>(workspace) + wl.plan + wl.carry;

    PrepArgs pa;
    pa.q = q; pa.k = k; pa.v = v; pa.beta = beta; pa.gate = gate;
    pa.chunk_tok0 = d;
    pa.chunk_len = d + n_chunks;
    pa.chunk_emit_slot = d + 2 * (int64_t)n_chunks;
    pa.req_chunk_cu = d + 3 * (int64_t)n_chunks;
    pa.ws_units = nullptr;   // set per slab
    pa.slab_begin = 0;
    pa.R = wl.R;
    pa.n_req = n_req;
    pa.L = s.L; pa.H_qk = s.H_qk; pa.H_v = s.H_v;
    pa.T_alloc = s.T_alloc;
    pa.scale = s.scale;
    pa.host_pool = nullptr; pa.host_slot_stride = 0; pa.staged_slot = nullptr; pa.staging = nullptr;
    pa.slot_elems = 0; pa.n_staged = 0; pa.n_copy_wgs = 0;

    RecurArgs ra;
    ra.o = o; ra.ws_units = nullptr;
    ra.carry = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + wl.plan);
    ra.slab_begin = 0;
    ra.R = wl.R;
    ra.req_chunk_cu = d + 3 * (int64_t)n_chunks;
    ra.req_src_slot = ra.req_chunk_cu + (n_req + 1);
    ra.req_order = ra.req_src_slot + n_req;
    ra.state_src = state_src; ra.state_dst = state_dst;
    ra.src_slot_stride = src_slot_stride; ra.dst_slot_stride = dst_slot_stride;
    ra.L = s.L; ra.H_qk = s.H_qk; ra.H_v = s.H_v;
    ra.T_alloc = s.T_alloc;
    ra.scale = s.scale;
    ra.o_bf16 = s.o_dtype == GDN_BF16;

    // ---- host tier: the start states go to the staging area.  If the pool is device-accessible
    //      pinned memory, workgroups appended to the first preparation launch fetch them over
    //      PCIe while that launch computes (only the recurrence needs them); otherwise they are
    //      copied on the caller's stream ahead of the first launch.  (Sending them over a second
    //      stream was measured: the two cross-stream event waits cost more than the 27 us copy
    //      of a 1 MiB state they hide.)
    if (src_on_host && n_staged > 0) {
        float* staging = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + staging_off);
        hipPointerAttribute_t attr;
        std::memset(&attr, 0, sizeof attr);
        const bool mapped = hipPointerGetAttributes(&attr, state_src) == hipSuccess && attr.type == hipMemoryTypeHost &&
                            attr.devicePointer != nullptr;
        if (!mapped) (void)hipGetLastError();   // an unregistered pointer is not an error here
        if (mapped && !use_fused) {
            pa.host_pool = static_cast<const float*>(attr.devicePointer);
            pa.host_slot_stride = src_slot_stride;
            pa.staged_slot = ra.req_order + n_req;
            pa.staging = staging;
            pa.slot_elems = slot_elems;
            pa.n_staged = n_staged;
            pa.n_copy_wgs = 32;
        } else {
            int32_t at = 0;
            for (int32_t r = 0; r < n_req; ++r) {
                if (src_slot[r] < 0) continue;
                const hipError_t e = hipMemcpyAsync(staging + (int64_t)at * slot_elems,
                                                    state_src + (int64_t)src_slot[r] * src_slot_stride,
                                                    (size_t)slot_elems * sizeof(float), hipMemcpyHostToDevice, stream);
                if (e != hipSuccess) return hip_err(e);
                ++at;
            }
        }
        ra.state_src = staging;
        ra.src_slot_stride = slot_elems;
    }

    // ---- many chains: preparation and recurrence fused, no operand image in memory
    if (use_fused) {
        FusedArgs fa;
        fa.q = q; fa.k = k; fa.v = v; fa.beta = beta; fa.gate = gate; fa.o = o;
        fa.chunk_tok0 = pa.chunk_tok0; fa.chunk_len = pa.chunk_len; fa.chunk_emit_slot = pa.chunk_emit_slot;
        fa.req_chunk_cu = ra.req_chunk_cu; fa.req_src_slot = ra.req_src_slot; fa.req_order = ra.req_order;
        fa.state_src = ra.state_src; fa.state_dst = state_dst;   // (the staging area when the pool is on the host)
        fa.src_slot_stride = ra.src_slot_stride; fa.dst_slot_stride = dst_slot_stride;
        const int gv = fused_heads_per_wg(s, (int64_t)n_chunks * s.L * s.H_v, plan.max_chunks_per_req);
        int32_t n_live = 0;          // requests with tokens: they come first in the order, and only they have chains
        for (int32_t r = 0; r < n_req; ++r) n_live += plan.req_chunk_cu[r + 1] > plan.req_chunk_cu[r];
        fa.n_chains = (int32_t)((int64_t)n_live * s.L * s.H_v / gv);
        fa.next_chain = reinterpret_cast<int32_t*>(workspace) + (3 * (int64_t)n_chunks + 4 * (int64_t)n_req + 1);
        fa.L = s.L; fa.H_qk = s.H_qk; fa.H_v = s.H_v;
        fa.T_alloc = s.T_alloc;
        fa.scale = s.scale;
        fa.o_bf16 = s.o_dtype == GDN_BF16;
        ProfChain prof(stream);
        const int per_cu = fused_wgs_per_cu(s, gv, (int64_t)n_chunks * s.L * s.H_v, plan.max_chunks_per_req);
        const hipError_t e = launch_fused(fa, s.d_k, gv, per_cu, stream);
        if (e != hipSuccess) return hip_err(e);
        prof.mark(1);
        std::lock_guard<std::mutex> lock(g_prof.mu);
        if (g_prof.on) g_prof.calls += 1;
        return GDN_OK;
    }

    const int32_t mc = plan.max_chunks_per_req;
    if (s.in_dtype == GDN_F32) return launch_all<float, 64, 64>(s, pa, ra, n_req, mc, slab_base, wl.slab, wl.n_bufs, stream);
    if (s.d_k == 64) return launch_all<half_t, 64, 64>(s, pa, ra, n_req, mc, slab_base, wl.slab, wl.n_bufs, stream);
    return launch_all<half_t, 128, 128>(s, pa, ra, n_req, mc, slab_base, wl.slab, wl.n_bufs, stream);
}

int32_t gdn_resume_prefill(const gdn_shape* shape, const void* q, const void* k, const void* v, const void* beta,
                           const void* gate, int32_t n_req, const int32_t* cu_seqlens, const int32_t* start_pos,
                           const float* state_src, int64_t src_slot_stride, int32_t src_n_slots,
                           const int32_t* src_slot, const int32_t* emit_cu, const int32_t* emit_pos,
                           float* state_dst, int64_t dst_slot_stride, int32_t dst_n_slots, const int32_t* emit_slot,
                           void* o, void* workspace, int64_t workspace_bytes, void* stream) {
    return prefill_impl(shape, q, k, v, beta, gate, n_req, cu_seqlens, start_pos, state_src, src_slot_stride, src_n_slots,
                        src_slot, emit_cu, emit_pos, state_dst, dst_slot_stride, dst_n_slots, emit_slot, o, workspace,
                        workspace_bytes, stream, POOL_DEVICE);
}

int32_t gdn_resume_prefill_static(const gdn_shape* shape, const void* q, const void* k, const void* v, const void* beta,
                                  const void* gate, int32_t n_req, const int32_t* cu_seqlens, const int32_t* start_pos,
                                  const float* state_src, int64_t src_slot_stride, int32_t src_n_slots,
                                  const int32_t* src_slot, const int32_t* emit_cu, const int32_t* emit_pos,
                                  float* state_dst, int64_t dst_slot_stride, int32_t dst_n_slots, const int32_t* emit_slot,
                                  void* o, void* stream) {
    return prefill_impl(shape, q, k, v, beta, gate, n_req, cu_seqlens, start_pos, state_src, src_slot_stride, src_n_slots,
                        src_slot, emit_cu, emit_pos, state_dst, dst_slot_stride, dst_n_slots, emit_slot, o, nullptr, 0,
                        stream, POOL_DEVICE_STATIC);
}

int64_t gdn_static_plan_capacity(void) { return STATIC_SCRATCH_BYTES; }


int32_t gdn_resume_prefill_host(const gdn_shape* shape, const void* q, const void* k, const void* v, const void* beta,
                                const void* gate, int32_t n_req, const int32_t* cu_seqlens, const int32_t* start_pos,
                                const float* host_state_src, int64_t src_slot_stride, int32_t src_n_slots,
                                const int32_t* src_slot, const int32_t* emit_cu, const int32_t* emit_pos,
                                float* state_dst, int64_t dst_slot_stride, int32_t dst_n_slots, const int32_t* emit_slot,
                                void* o, void* workspace, int64_t workspace_bytes, void* stream) {
    return prefill_impl(shape, q, k, v, beta, gate, n_req, cu_seqlens, start_pos, host_state_src, src_slot_stride,
                        src_n_slots, src_slot, emit_cu, emit_pos, state_dst, dst_slot_stride, dst_n_slots, emit_slot, o,
                        workspace, workspace_bytes, stream, POOL_HOST);
}

int64_t gdn_workspace_bytes_host(const gdn_shape* shape, int32_t n_req, int64_t total_tokens, int32_t n_emit) {
    const int64_t base = gdn_workspace_bytes(shape, n_req, total_tokens, n_emit);
    if (base < 0) return base;
    const int64_t slot_bytes = (int64_t)shape->L * shape->H_v * shape->d_v * shape->d_k * (int64_t)sizeof(float);
    return align_up(base, 256) + (int64_t)n_req * slot_bytes;
}

int32_t ckpt_fetch_host(const float* host_pool, int64_t host_slot_stride, int32_t host_n_slots, const int32_t* host_ids,
                        float* dev_pool, int64_t dev_slot_stride, int32_t dev_n_slots, const int32_t* dev_ids, int32_t n,
                        int64_t state_elems, void* stream) {
    const int32_t rc = check_tier_args(host_pool, host_slot_stride, host_n_slots, host_ids, dev_pool, dev_slot_stride,
                                       dev_n_slots, dev_ids, n, state_elems);
    if (rc != GDN_OK || n == 0 || state_elems == 0) return rc;
    std::vector<int32_t> sorted(dev_ids, dev_ids + n);
    std::sort(sorted.begin(), sorted.end());
    if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return GDN_ERR_SLOT_DUP;
    for (int32_t i = 0; i < n; ++i) {
        const hipError_t e = hipMemcpyAsync(dev_pool + (int64_t)dev_ids[i] * dev_slot_stride,
                                            host_pool + (int64_t)host_ids[i] * host_slot_stride,
                                            (size_t)state_elems * sizeof(float), hipMemcpyHostToDevice, (hipStream_t)stream);
        if (e != hipSuccess) return hip_err(e);
    }
    return GDN_OK;
}

int32_t ckpt_spill_host(float* host_pool, int64_t host_slot_stride, int32_t host_n_slots, const int32_t* host_ids,
                        const float* dev_pool, int64_t dev_slot_stride, int32_t dev_n_slots, const int32_t* dev_ids, int32_t n,
                        int64_t state_elems, void* stream) {
    const int32_t rc = check_tier_args(host_pool, host_slot_stride, host_n_slots, host_ids, dev_pool, dev_slot_stride,
                                       dev_n_slots, dev_ids, n, state_elems);
    if (rc != GDN_OK || n == 0 || state_elems == 0) return rc;
    std::vector<int32_t> sorted(host_ids, host_ids + n);
    std::sort(sorted.begin(), sorted.end());
    if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return GDN_ERR_SLOT_DUP;
    for (int32_t i = 0; i < n; ++i) {
        const hipError_t e = hipMemcpyAsync(host_pool + (int64_t)host_ids[i] * host_slot_stride,
                                            dev_pool + (int64_t)dev_ids[i] * dev_slot_stride,
                                            (size_t)state_elems * sizeof(float), hipMemcpyDeviceToHost, (hipStream_t)stream);
        if (e != hipSuccess) return hip_err(e);
    }
    return GDN_OK;
}

int32_t gdn_decode_step(const gdn_shape* shape, const void* q, const void* k, const void* v, const void* beta,
                        const void* gate, int32_t n_req, float* pool, int64_t slot_stride, int32_t n_slots,
                        const int32_t* slot, void* o, void* stream_) {
    int32_t rc = check_shape(shape);
    if (rc != GDN_OK) return rc;
    const gdn_shape& s = *shape;
    if (n_req < 0 || n_slots < 0) return GDN_ERR_COUNT;
    if (n_req == 0) return GDN_OK;
    if (n_req > s.T_alloc) return GDN_ERR_SEQLENS;
    if (!q || !k || !v || !beta || !gate || !pool || !slot || !o) return GDN_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(pool) || (slot_stride & 3))
        return GDN_ERR_ALIGN;
    const int64_t slot_elems = (int64_t)s.L * s.H_v * s.d_v * s.d_k;
    if (slot_stride < slot_elems) return GDN_ERR_SHAPE;
    {
        std::vector<int32_t> sorted(slot, slot + n_req);
        std::sort(sorted.begin(), sorted.end());
        if (sorted.front() < 0 || sorted.back() >= n_slots) return GDN_ERR_SLOT_RANGE;
        if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return GDN_ERR_SLOT_DUP;
    }
    hipStream_t stream = (hipStream_t)stream_;
    DecodeArgs a;
    a.q = q; a.k = k; a.v = v; a.beta = beta; a.gate = gate;
    a.pool = pool; a.o = o;
    a.slot_stride = slot_stride; a.T_alloc = s.T_alloc;
    a.L = s.L; a.H_qk = s.H_qk; a.H_v = s.H_v;
    a.scale = s.scale;
    a.o_bf16 = s.o_dtype == GDN_BF16;
    // states beyond half of the 256 MiB memory-side cache will not be there for the next step: stream them
    const bool stream_states = (int64_t)n_req * slot_elems * (int64_t)sizeof(float) > ((int64_t)128 << 20);
    for (int32_t base = 0; base < n_req; base += DECODE_IDS) {
        const int32_t m = std::min(DECODE_IDS, n_req - base);
        DecodeIds ids;
        std::memset(&ids, 0, sizeof ids);
        std::memcpy(ids.slot, slot + base, sizeof(int32_t) * m);
        a.req_base = base;
        const dim3 grid((unsigned)(s.d_v / 32), (unsigned)(s.L * s.H_v), (unsigned)m);
        if (s.in_dtype == GDN_F32) {
            if (stream_states) hipLaunchKernelGGL((gdn_decode_kernel<float, 64, 64, true>), grid, dim3(256), 0, stream, a, ids);
            else hipLaunchKernelGGL((gdn_decode_kernel<float, 64, 64, false>), grid, dim3(256), 0, stream, a, ids);
        } else if (s.d_k == 64) {
            if (stream_states) hipLaunchKernelGGL((gdn_decode_kernel<half_t, 64, 64, true>), grid, dim3(256), 0, stream, a, ids);
            else hipLaunchKernelGGL((gdn_decode_kernel<half_t, 64, 64, false>), grid, dim3(256), 0, stream, a, ids);
        } else {
            if (stream_states) hipLaunchKernelGGL((gdn_decode_kernel<half_t, 128, 128, true>), grid, dim3(256), 0, stream, a, ids);
            else hipLaunchKernelGGL((gdn_decode_kernel<half_t, 128, 128, false>), grid, dim3(256), 0, stream, a, ids);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_err(e);
    }
    return GDN_OK;
}

}  // extern "C"
