// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <exception>
#include <functional>
#include <new>
#include <vector>

#include "apm.h"

namespace apm {

// ---- errors -------------------------------------------------------------------------------
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Every int-returning entry point runs inside this: no C++ exception crosses the C boundary.
template <class F>
int guarded(F&& f) noexcept {
    try {
        return f();
    } catch (const std::bad_alloc&) {
        return fail(APM_ENOMEM, "out of host memory");
    } catch (const std::exception& e) {
        return fail(APM_EDEVICE, "unexpected failure: %s", e.what());
    } catch (...) {
        return fail(APM_EDEVICE, "unexpected failure");
    }
}

#define APM_HIP(expr)                                                                   \
    do {                                                                                \
        hipError_t apm_e_ = (expr);                                                     \
        if (apm_e_ != hipSuccess)                                                       \
            return ::apm::fail(APM_EDEVICE, "%s failed: %s", #expr, hipGetErrorString(apm_e_)); \
    } while (0)

// ---- packing plan -------------------------------------------------------------------------
constexpr int64_t kAlign = 8;  // elements; keeps 128-bit accesses aligned for both widths

struct PageEntry {
    int64_t used = 0;
    int32_t n_tensors = 0;
    int64_t tensor[2] = {-1, -1};  // index in the tensor list
    int64_t tensor_elems[2] = {0, 0};
};

struct Plan {
    int64_t E = 0;
    int64_t total = 0;
    std::vector<apm_segment> segs;
    std::vector<PageEntry> pages;
};

int make_plan(int64_t E, const int64_t* numels, int64_t n, Plan* out);
int emit_plan(const Plan& plan, apm_segment* segs, int64_t* n_segs, int64_t* n_pages,
              double* fragmentation);

inline int elem_bytes(int state) { return state <= APM_V32 ? 4 : 2; }

// ---- pinned staging ring: small host arrays (page lists, copy descriptors) to the device ----
struct StageRing {
    static constexpr int K = 8;
    void* h[K] = {};
    void* d[K] = {};
    size_t cap[K] = {};
    hipEvent_t ev[K] = {};
    bool busy[K] = {};
    int next = 0;
    // Returns a slot whose previous use has completed, with at least `bytes` capacity.
    int acquire(size_t bytes, int* slot);
    // Copies the first `bytes` of the slot's host buffer to its device buffer on `s`.
    int commit(int slot, size_t bytes, hipStream_t s);
    // To be called after the kernels that read the slot's device buffer have been enqueued on `s`:
    // the slot is not handed out again before they have run (commit alone only covers the copy).
    int seal(int slot, hipStream_t s);
    void destroy();
};

// ---- kernels ------------------------------------------------------------------------------
constexpr int kReduceTile = 16384;  // gradient elements per workgroup of the reduce kernel

// Per-page view of the tenant tensors, for kernels that read gradients from / write bf16
// parameters to the caller's contiguous tensors directly instead of the G16 / P16 page classes.
// Tenant k covers page elements [off[k], off[k]+n[k]); g[k] / q[k] point at the tensor element
// that sits at off[k].  off[k] is a multiple of 8 and the pointers are 16-byte aligned.
struct PageSegs {
    int32_t off[2];
    int32_t n[2];
    const uint16_t* g[2];
    uint16_t* q[2];
};

// What one listed page needs in the update kernel, gathered into one 32-byte record so that a
// workgroup fetches it with a single scalar load: written per call by the finalize kernel (after a
// reduce pass) or by the prepare kernel (no reduce pass).
struct PageMeta {
    int32_t used;   // used extent of the page (elements)
    float scale;    // clip scale; negative = the page is skipped
    int64_t gpage;  // page index for the 16-bit classes (and the page table)
    int64_t spage;  // page index for the fp32 classes
    int64_t pad;
};

// The listed pages of one call, grouped by used extent: the pages of a class sit at consecutive
// list positions and are launched together, with a grid sized for the class's largest extent, so
// that a nearly empty page (a small tensor alone in its page) does not cost a full page's worth
// of workgroups that only find out they have nothing to do.
// Wavefronts of the update kernel when it reads and writes fp32 classes in host memory across
// PCIe (the streamer's direct mode, the file tier's window); see apm_stream.hip for the sweep.
constexpr int kDirectWavefronts = 48;

constexpr int kMaxExtentClasses = 4;
struct ExtentClass {
    int64_t begin;     // first list position
    int64_t count;     // pages
    int64_t max_used;  // largest used extent among them (elements)
};

struct AdamwLaunch {
    float* p32;
    float* m32;
    float* v32;
    const uint16_t* g16;
    uint16_t* p16;
    const int32_t* used;          // device, indexed by grad page id
    const PageSegs* segs;         // device, indexed like the page list; needed if gather or scatter
    PageMeta* meta;               // device scratch, [n_listed], filled by the reduce / prepare pass
    bool gather;                  // read g from the tenant tensors (segs[].g) instead of g16
    bool scatter;                 // write p16 to the tenant tensors (segs[].q) instead of p16
    const int64_t* state_pages;   // device list or nullptr (then state_first + i)
    const int64_t* grad_pages;    // device list or nullptr (then grad_first + i)
    int64_t state_first;
    int64_t grad_first;
    int64_t n_listed;
    ExtentClass cls[kMaxExtentClasses];  // n_cls == 0: one class, all positions, extent E
    int n_cls;
    const int32_t* out_index;     // device: list position -> index into grad_norm / skip_mask;
                                  // nullptr = the position itself
    int64_t E;
    double* partials;             // [n_listed][S] per-slice sums of squares; nullptr = no reduce pass
    uint32_t* nzflags;            // [n_listed][S] per-slice OR of magnitude bits
    int32_t S;                    // slices per page = ceil(E / kReduceTile)
    float* grad_norm;             // device, nullable
    uint8_t* skip_mask;           // device, nullable
    float b1, omb1, b2, omb2, inv_sqrt_bc2, eps, step_size, lr_wd;
    double max_norm;
    int32_t skip_mode;
    int32_t stride_wavefronts;    // > 0: the update runs as that many wavefronts striding over all
                                  // page slices (fp32 classes in host memory); 0: one per slice
    int32_t stride_waves_per_wg;  // how many of them share a workgroup, 1..16
    bool host_write_through;      // stride form: fp32 state stores written through at system scope
};

// Reduce pass (fills meta with clip scale / skip); or, when no reduce pass is needed, the prepare
// pass (fills meta with scale 1).  One of the two must precede launch_adamw on the same stream.
hipError_t launch_grad_reduce(const AdamwLaunch& a, hipStream_t s);
hipError_t launch_prepare(const AdamwLaunch& a, hipStream_t s);
hipError_t launch_adamw(const AdamwLaunch& a, hipStream_t s);
hipError_t launch_grad_accum(uint16_t* acc, const uint16_t* g16, const int32_t* used,
                             const int64_t* d_pages, int64_t first, int64_t n_listed, int64_t E,
                             hipStream_t s);

struct SegDesc {
    const void* src;
    void* dst;
    int64_t nbytes;
};
hipError_t launch_seg_copy(const SegDesc* d_descs, int64_t n, int64_t max_bytes, hipStream_t s);

// One kernel that moves an incoming batch (3 fp32 classes, in_bytes each, host -> staging) and an
// outgoing batch (out_bytes each, staging -> host) at once; either byte count may be 0.  All
// addresses are device-side addresses, 16-byte aligned; byte counts are multiples of 16.
struct DuplexCopy {
    const char* in_src[3];
    char* in_dst[3];
    const char* out_src[3];
    char* out_dst[3];
    int64_t in_bytes, out_bytes;
    // Optional: move only the used extent of each page.  used = the device page table (elements per
    // page), *_first_page = the table index of each batch's first page, page_bytes = E * 4.
    const int32_t* used;
    int64_t in_first_page, out_first_page, page_bytes;
    uint32_t items_per_page;  // filled in by launch_duplex_copy
    int host_store_policy;    // stores to the host pages: 0 non-temporal, 3 written through at system scope
};
hipError_t launch_duplex_copy(const DuplexCopy& d, int wavefronts, int per_wg, hipStream_t s);

// Fills the scalar fields of `a` from the hyper-parameters (all derived in double, rounded once).
int prepare_hyper(const apm_hyper* h, int64_t step, AdamwLaunch* a);

}  // namespace apm

struct apm_pool {
    apm_pool_desc desc{};
    void* base[APM_N_STATES] = {};
    void* alloc[APM_N_STATES] = {};  // what the library allocated for the class (base = alloc + skew)
    bool owned[APM_N_STATES] = {};

    bool has_layout = false;
    std::vector<int64_t> layout_numels;
    std::vector<int64_t> layout_ids;
    apm::Plan plan;

    int fd[APM_N_STATES] = {-1, -1, -1, -1, -1};  // FILE pools: one file per stored class

    int32_t* d_used = nullptr;      // device page table: used extent per page
    double* d_partials = nullptr;   // reduce scratch, n_pages * S
    uint32_t* d_nzflags = nullptr;
    apm::PageMeta* d_meta = nullptr;  // n_pages entries
    int32_t S = 0;
    apm::StageRing ring;

    // one-step-stale update state
    hipStream_t upd_stream = nullptr;
    bool upd_overlaps = false;  // measured: its kernels run beside the producer stream's
    uint16_t* gbuf[2] = {nullptr, nullptr};
    hipEvent_t ev_staged[2] = {};
    hipEvent_t ev_applied[2] = {};
    bool applied_valid[2] = {false, false};
    hipEvent_t ev_flush = nullptr;
    int cur = 0;
    bool buffered = false;
    int64_t applied = 0;
    // What the buffered gradient was handed over with: it is applied, one call later, with the
    // hyper-parameters and the page list of the call that brought it.
    apm_hyper buf_hyper{};
    std::vector<int64_t> buf_pages;  // copy of the caller's list (unused if buf_pages_null)
    bool buf_pages_null = true;      // the call listed pages [0, buf_n_pages)
    int64_t buf_n_pages = 0;
    float* delayed_norm = nullptr;
    uint8_t* delayed_skip = nullptr;

    // kernel timing (measurement aid)
    bool timing = false;
    struct TimedLaunch { int cls; hipEvent_t begin, end; };
    std::vector<TimedLaunch> timed;

    bool stores(int s) const { return s >= 0 && s < APM_N_STATES && (desc.state_mask >> s) & 1u; }
};

namespace apm {
// Validates a page list and enqueues the two kernels of one step.  g16_override != nullptr
// replaces the pool's G16 region as the gradient source.
int enqueue_step(apm_pool* pool, const int64_t* pages, int64_t n_pages, int64_t step,
                 const apm_hyper* hyper, const uint16_t* g16_override, float* grad_norm,
                 uint8_t* skip_mask, hipStream_t stream, const apm_tensor* grad_tensors = nullptr,
                 const apm_tensor* p16_tensors = nullptr, int64_t n_tensors = 0);
int ensure_scratch(apm_pool* pool);
// Allocates the ping-pong gradient halves, the events and the update stream of the delayed path.
// caller != nullptr-able: the stream the producer works on; the update stream is chosen so that
// its kernels run beside that stream's (see make_overlapping_stream).
int ensure_delayed(apm_pool* pool, hipStream_t caller, bool probe);

// Whether kernels on two streams of one process run at the same time is not something the API
// states: the runtime maps streams onto a few hardware queues, and work of two streams that share
// a queue runs in order.  These helpers measure it with two short spin kernels (a few hundred
// microseconds each; both streams are synchronised first).
int streams_overlap(hipStream_t a, hipStream_t b, bool* out);
// A new non-blocking stream whose kernels overlap with those of `with` (and of `*also`, if given);
// tries a few candidates and keeps the last one (*overlaps = false) if none does.
int make_overlapping_stream(hipStream_t with, hipStream_t* out, bool* overlaps, const hipStream_t* also = nullptr);
// FILE <-> HOST page copy (synchronous).
int file_page_copy(apm_pool* dst, int64_t dst_page, apm_pool* src, int64_t src_page, int64_t n_pages,
                   int state, hipStream_t stream);

// The one-step-stale hand-over shared by apm_step_delayed and the streamer's delayed step:
// applies the buffered gradient through `apply` (which enqueues one update reading the gradient
// half it is given, with the step number, page list and hyper-parameters it is given -- those of
// the call that handed that gradient over -- on the pool's update stream), then stages new_g16
// into the other half on `caller` together with this call's page list and hyper-parameters
// (nullptr = flush).
using DelayedApply = std::function<int(const uint16_t* g16, int64_t step, hipStream_t upd_stream,
                                       const int64_t* pages, int64_t n_pages, const apm_hyper* hyper)>;
int delayed_call(apm_pool* pool, const int64_t* pages, int64_t n_pages, const void* new_g16,
                 const apm_hyper* hyper, hipStream_t caller, const DelayedApply& apply);

// Brackets one kernel launch with events when the pool's timing is on.
struct ScopedTiming {
    apm_pool* pool;
    hipStream_t stream;
    hipEvent_t end = nullptr;
    ScopedTiming(apm_pool* p, int cls, hipStream_t s) : pool(p), stream(s) {
        if (!p->timing) return;
        hipEvent_t b = nullptr;
        if (hipEventCreate(&b) != hipSuccess || hipEventCreate(&end) != hipSuccess) { end = nullptr; return; }
        (void)hipEventRecord(b, s);
        p->timed.push_back({cls, b, end});
    }
    ~ScopedTiming() { if (end) (void)hipEventRecord(end, stream); }
};
}  // namespace apm
