// apm_page_adamw_step_noalloc: the resident step for callers that cannot allocate (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc).  It launches the same
// reduce / finalize / update kernels as apm_page_adamw_step, but the per-page scratch they need
// (page records, per-slice sums of squares, per-slice non-zero flags) lives in a fixed device
// array owned by the library instead of buffers the pool allocates on first use, and nothing on
// its path allocates: no hipMalloc / hipFree, no events, no staging ring, no host containers.
#include <mutex>

#include "apm_internal.h"

// Fixed scratch, one copy per GPU the library runs on (held until the process ends).
// No `used` attribute here: the compiler gives a static device variable that host code refers to
// an externally visible symbol in the code object, which is what the runtime's symbol lookup
// needs; with the attribute it stays a local symbol and the lookup below cannot find it.
constexpr size_t kScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace apm {
namespace {

// In host code `scratch` is only a handle for the symbol, not a device address.  Its address on a
// GPU is asked for once per device, with that device current, and kept here; host code passes
// this pointer -- never the array's name -- to the kernels.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int scratch_for_device(int hip_device, unsigned char** out) {
    if (hip_device < 0 || hip_device >= kMaxDevices) return fail(APM_EDEVICE, "device ordinal %d is beyond the %d devices the fixed scratch is resolved for", hip_device, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[hip_device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // the current device's copy
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(APM_EDEVICE, "hipGetSymbolAddress(scratch) failed on device %d: %s", hip_device, hipGetErrorString(e));
        }
        g_scratch_ptr[hip_device] = p;
    }
    *out = static_cast<unsigned char*>(g_scratch_ptr[hip_device]);
    return APM_OK;
}

constexpr size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace
}  // namespace apm

using namespace apm;

extern "C" size_t apm_noalloc_scratch_bytes(void) { return kScratchBytes; }

extern "C" int64_t apm_noalloc_max_pages(int64_t page_elems) {
    if (page_elems <= 0) return 0;
    const int64_t S = (page_elems + kReduceTile - 1) / kReduceTile;
    // three 256-byte aligned sections: records, sums, flags
    const int64_t per_page = (int64_t)sizeof(PageMeta) + S * (int64_t)(sizeof(double) + sizeof(uint32_t));
    return ((int64_t)kScratchBytes - 3 * 256) / per_page;
}

extern "C" int apm_page_adamw_step_noalloc(apm_pool* pool, int64_t n_pages, int64_t step,
                                           const apm_hyper* hyper, float* grad_norm,
                                           uint8_t* skip_mask, void* stream) {
    return apm::guarded([&]() -> int {
        if (!pool) return fail(APM_EINVAL, "NULL pool");
        if (pool->desc.device != APM_DEV_GPU) return fail(APM_EDEVICE, "the update runs on GPU pools only");
        for (int st = 0; st < APM_N_STATES; ++st)
            if (!pool->stores(st)) return fail(APM_ESTATE, "pool does not store state class %d", st);
        if (n_pages < 0 || n_pages > pool->desc.n_pages) return fail(APM_ERANGE, "page count %lld out of range", (long long)n_pages);
        AdamwLaunch L{};
        int rc = prepare_hyper(hyper, step, &L);
        if (rc != APM_OK) return rc;
        const int64_t max_pages = apm_noalloc_max_pages(pool->desc.page_elems);
        if (n_pages > max_pages)
            return fail(APM_ERANGE, "%lld pages of %lld elements need more than the %zu-byte fixed scratch (at most %lld pages of this size): use apm_page_adamw_step",
                        (long long)n_pages, (long long)pool->desc.page_elems, kScratchBytes, (long long)max_pages);
        if (n_pages == 0) return APM_OK;
        APM_HIP(hipSetDevice(pool->desc.hip_device));
        unsigned char* base = nullptr;
        rc = scratch_for_device(pool->desc.hip_device, &base);
        if (rc != APM_OK) return rc;

        // Carve the scratch: page records, per-slice sums, per-slice flags.  Nothing needs clearing:
        // the reduce pass writes every slice entry the finalize pass reads (slice 0 of a page
        // always, the others whenever they hold used elements) and the finalize / prepare pass
        // writes every listed page's record before the update reads it.
        const size_t S = (size_t)pool->S;
        const size_t n = (size_t)n_pages;
        L.meta = reinterpret_cast<PageMeta*>(base);
        size_t at = round256(n * sizeof(PageMeta));
        L.partials = reinterpret_cast<double*>(base + at);
        at += round256(n * S * sizeof(double));
        L.nzflags = reinterpret_cast<uint32_t*>(base + at);
        at += n * S * sizeof(uint32_t);
        if (at > kScratchBytes) return fail(APM_ERANGE, "fixed scratch too small");  // cannot happen after the check above

        L.p32 = static_cast<float*>(pool->base[APM_P32]);
        L.m32 = static_cast<float*>(pool->base[APM_M32]);
        L.v32 = static_cast<float*>(pool->base[APM_V32]);
        L.g16 = static_cast<const uint16_t*>(pool->base[APM_G16]);
        L.p16 = static_cast<uint16_t*>(pool->base[APM_P16]);
        L.used = pool->d_used;
        L.n_listed = n_pages;  // pages [0, n_pages) in order: no list, no output permutation,
        L.n_cls = 0;           // one launch geometry sized for full pages
        L.E = pool->desc.page_elems;
        L.S = pool->S;
        L.grad_norm = grad_norm;
        L.skip_mask = skip_mask;
        hipStream_t s = static_cast<hipStream_t>(stream);
        const bool need_reduce = grad_norm || skip_mask || L.max_norm > 0.0 || L.skip_mode != APM_SKIP_NONE;
        if (need_reduce) {
            APM_HIP(launch_grad_reduce(L, s));
        } else {
            L.partials = nullptr;
            L.nzflags = nullptr;
            APM_HIP(launch_prepare(L, s));
        }
        APM_HIP(launch_adamw(L, s));
        return APM_OK;
    });
}
