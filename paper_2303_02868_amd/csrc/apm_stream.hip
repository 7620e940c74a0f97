// Streamed update: fp32 master / momentum / variance pages live in pinned host memory and pass
// through a small ring of HBM staging slots, copy-in, update and copy-out each on its own stream
// so that the three overlap (Sec. 4.2: overlap movement with computation; Sec. 5 "Allocator":
// asynchronous page copies; the update is page-granular by Sec. 4.3's last paragraph).
//
// Mixed residency (Sec. 4.2, the GPU cache of optimizer states): the first R pages may keep their
// fp32 classes in a GPU pool; they are updated in place, in chunks interleaved with the streamed
// batches on the compute stream, and only pages [R, N) cross PCIe.
//
// Slot life cycle for batch b (slot = b mod n_slots):
//   copy-in : wait D2H(b - n_slots) -> H2D p,m,v           -> record h2d[slot]
//   compute : wait h2d[slot]        -> reduce + update      -> record cmp[slot]
//   copy-out: wait cmp[slot]        -> D2H p,m,v            -> record d2h[slot]
// Streams are in order, so these three edges are the only synchronisation needed.
#include "apm_internal.h"

struct apm_streamer {
    apm_pool* host = nullptr;
    apm_pool* dev = nullptr;
    apm_pool* cache = nullptr;  // optional GPU pool holding the fp32 classes of pages [0, R)
    int64_t R = 0;              // number of leading pages whose fp32 state is HBM-resident
    int64_t B = 0;
    int n_slots = 0;
    float* stage[3] = {nullptr, nullptr, nullptr};  // each n_slots * B * E floats
    hipStream_t s_in = nullptr, s_cmp = nullptr, s_out = nullptr;
    std::vector<hipEvent_t> ev_h2d, ev_cmp, ev_d2h;
    hipEvent_t ev_start = nullptr, ev_done = nullptr;
};

using namespace apm;

namespace {
void free_streamer(apm_streamer* s) {
    for (hipStream_t st : {s->s_in, s->s_cmp, s->s_out})
        if (st) { (void)hipStreamSynchronize(st); (void)hipStreamDestroy(st); }
    for (auto* v : {&s->ev_h2d, &s->ev_cmp, &s->ev_d2h})
        for (hipEvent_t e : *v) if (e) (void)hipEventDestroy(e);
    if (s->ev_start) (void)hipEventDestroy(s->ev_start);
    if (s->ev_done) (void)hipEventDestroy(s->ev_done);
    for (float* p : s->stage) if (p) (void)hipFree(p);
    delete s;
}
}  // namespace

extern "C" int apm_streamer_create(apm_streamer** out, apm_pool* host, apm_pool* dev,
                                   int64_t batch_pages, int n_slots) {
    if (!out || !host || !dev) return fail(APM_EINVAL, "NULL argument");
    if (host->desc.device != APM_DEV_HOST || dev->desc.device != APM_DEV_GPU) return fail(APM_EDEVICE, "expected a HOST pool and a GPU pool");
    for (int st : {APM_P32, APM_M32, APM_V32}) if (!host->stores(st)) return fail(APM_ESTATE, "host pool lacks fp32 class %d", st);
    for (int st : {APM_G16, APM_P16}) if (!dev->stores(st)) return fail(APM_ESTATE, "GPU pool lacks 16-bit class %d", st);
    if (host->desc.page_elems != dev->desc.page_elems) return fail(APM_EINVAL, "pools have different page sizes");
    if (host->desc.n_pages < dev->desc.n_pages) return fail(APM_EINVAL, "host pool has fewer pages than the GPU pool");
    if (batch_pages < 1 || batch_pages > dev->desc.n_pages) return fail(APM_EINVAL, "batch_pages out of range");
    if (n_slots < 2 || n_slots > 64) return fail(APM_EINVAL, "n_slots must be in [2, 64]");
    APM_HIP(hipSetDevice(dev->desc.hip_device));
    apm_streamer* s = new apm_streamer();
    s->host = host; s->dev = dev; s->B = batch_pages; s->n_slots = n_slots;
    const size_t bytes = (size_t)n_slots * (size_t)batch_pages * (size_t)dev->desc.page_elems * sizeof(float);
    hipError_t e = hipSuccess;
    for (int k = 0; k < 3 && e == hipSuccess; ++k) e = hipMalloc((void**)&s->stage[k], bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        free_streamer(s);
        return fail(APM_ENOMEM, "allocating 3 x %zu bytes of staging slots failed: %s", bytes, hipGetErrorString(e));
    }
    auto mk_stream = [&](hipStream_t* st) { return hipStreamCreateWithFlags(st, hipStreamNonBlocking); };
    auto mk_event = [&](hipEvent_t* ev) { return hipEventCreateWithFlags(ev, hipEventDisableTiming); };
    e = mk_stream(&s->s_in);
    if (e == hipSuccess) e = mk_stream(&s->s_cmp);
    if (e == hipSuccess) e = mk_stream(&s->s_out);
    s->ev_h2d.assign((size_t)n_slots, nullptr);
    s->ev_cmp.assign((size_t)n_slots, nullptr);
    s->ev_d2h.assign((size_t)n_slots, nullptr);
    for (int k = 0; k < n_slots && e == hipSuccess; ++k) {
        e = mk_event(&s->ev_h2d[(size_t)k]);
        if (e == hipSuccess) e = mk_event(&s->ev_cmp[(size_t)k]);
        if (e == hipSuccess) e = mk_event(&s->ev_d2h[(size_t)k]);
    }
    if (e == hipSuccess) e = mk_event(&s->ev_start);
    if (e == hipSuccess) e = mk_event(&s->ev_done);
    if (e != hipSuccess) {
        free_streamer(s);
        return fail(APM_EDEVICE, "creating streams/events failed: %s", hipGetErrorString(e));
    }
    int rc = ensure_scratch(dev);
    if (rc != APM_OK) { free_streamer(s); return rc; }
    *out = s;
    return APM_OK;
}

extern "C" int apm_streamer_destroy(apm_streamer* s) {
    if (!s) return APM_OK;
    (void)hipSetDevice(s->dev->desc.hip_device);
    free_streamer(s);
    return APM_OK;
}

namespace {
enum { kDoH2D = 1, kDoD2H = 2, kDoUpdate = 4 };

// The pipeline.  `what` selects its parts: the full step uses all three; the copy-only
// measurement entry point drops the kernels (and optionally one direction) but keeps the streams,
// the event structure and the copy sizes.
int run_pipeline(apm_streamer* s, int what, int64_t step, const apm_hyper* hyper, float* grad_norm,
                 uint8_t* skip_mask, void* stream) {
    apm_pool* dev = s->dev;
    apm_pool* host = s->host;
    if (!dev->has_layout) return fail(APM_ESTATE, "the GPU pool has no layout");
    AdamwLaunch L{};
    int rc = APM_OK;
    if (what & kDoUpdate) rc = prepare_hyper(hyper, step, &L);
    if (rc != APM_OK) return rc;
    APM_HIP(hipSetDevice(dev->desc.hip_device));
    hipStream_t caller = static_cast<hipStream_t>(stream);
    const int64_t N = (int64_t)dev->plan.pages.size();
    const int64_t E = dev->desc.page_elems;
    const size_t pb = (size_t)E * sizeof(float);

    APM_HIP(hipEventRecord(s->ev_start, caller));
    APM_HIP(hipStreamWaitEvent(s->s_in, s->ev_start, 0));
    APM_HIP(hipStreamWaitEvent(s->s_cmp, s->ev_start, 0));
    APM_HIP(hipStreamWaitEvent(s->s_out, s->ev_start, 0));

    L.g16 = static_cast<const uint16_t*>(dev->base[APM_G16]);
    L.p16 = static_cast<uint16_t*>(dev->base[APM_P16]);
    L.used = dev->d_used;
    L.E = E;
    L.S = dev->S;
    L.p32 = s->stage[0];
    L.m32 = s->stage[1];
    L.v32 = s->stage[2];
    const bool need_reduce = grad_norm || skip_mask || L.max_norm > 0.0 || L.skip_mode != APM_SKIP_NONE;
    if (need_reduce) {
        L.partials = dev->d_partials;
        L.nzflags = dev->d_nzflags;
        L.scale = dev->d_scale;
    }
    const int states[3] = {APM_P32, APM_M32, APM_V32};
    const int64_t R = s->cache ? (s->R < N ? s->R : N) : 0;
    const int64_t n_batches = (N - R + s->B - 1) / s->B;
    // resident pages are updated in n_batches chunks (one chunk if nothing is streamed)
    const int64_t chunk = n_batches > 0 ? (R + n_batches - 1) / n_batches : R;
    int64_t r_done = 0;
    auto resident_chunk = [&]() -> int {
        if (!(what & kDoUpdate) || r_done >= R) return APM_OK;
        const int64_t nr = R - r_done < chunk ? R - r_done : chunk;
        AdamwLaunch C = L;
        C.p32 = static_cast<float*>(s->cache->base[APM_P32]);
        C.m32 = static_cast<float*>(s->cache->base[APM_M32]);
        C.v32 = static_cast<float*>(s->cache->base[APM_V32]);
        C.state_first = C.grad_first = r_done;
        C.n_listed = nr;
        C.grad_norm = grad_norm ? grad_norm + r_done : nullptr;
        C.skip_mask = skip_mask ? skip_mask + r_done : nullptr;
        if (need_reduce) APM_HIP(launch_grad_reduce(C, s->s_cmp));
        APM_HIP(launch_adamw(C, s->s_cmp));
        r_done += nr;
        return APM_OK;
    };
    if (n_batches == 0) {
        rc = resident_chunk();
        if (rc != APM_OK) return rc;
        APM_HIP(hipEventRecord(s->ev_cmp[0], s->s_cmp));
        APM_HIP(hipStreamWaitEvent(s->s_out, s->ev_cmp[0], 0));
    }
    for (int64_t b = 0; b < n_batches; ++b) {
        const size_t slot = (size_t)(b % s->n_slots);
        const int64_t first = R + b * s->B;
        const int64_t nb = N - first < s->B ? N - first : s->B;
        const size_t slot_off = slot * (size_t)s->B * (size_t)E;  // floats
        if (b >= s->n_slots) APM_HIP(hipStreamWaitEvent(s->s_in, s->ev_d2h[slot], 0));
        for (int k = 0; k < 3 && (what & kDoH2D); ++k) {
            const char* src = static_cast<const char*>(host->base[states[k]]) + (size_t)first * pb;
            APM_HIP(hipMemcpyAsync(s->stage[k] + slot_off, src, pb * (size_t)nb, hipMemcpyHostToDevice, s->s_in));
        }
        APM_HIP(hipEventRecord(s->ev_h2d[slot], s->s_in));

        rc = resident_chunk();  // runs while this batch's copy-in is in flight
        if (rc != APM_OK) return rc;
        APM_HIP(hipStreamWaitEvent(s->s_cmp, s->ev_h2d[slot], 0));
        L.state_first = (int64_t)slot * s->B;
        L.grad_first = first;
        L.n_listed = nb;
        L.grad_norm = grad_norm ? grad_norm + first : nullptr;
        L.skip_mask = skip_mask ? skip_mask + first : nullptr;
        if (what & kDoUpdate) {
            if (need_reduce) APM_HIP(launch_grad_reduce(L, s->s_cmp));
            APM_HIP(launch_adamw(L, s->s_cmp));
        }
        APM_HIP(hipEventRecord(s->ev_cmp[slot], s->s_cmp));

        APM_HIP(hipStreamWaitEvent(s->s_out, s->ev_cmp[slot], 0));
        for (int k = 0; k < 3 && (what & kDoD2H); ++k) {
            char* dst = static_cast<char*>(host->base[states[k]]) + (size_t)first * pb;
            APM_HIP(hipMemcpyAsync(dst, s->stage[k] + slot_off, pb * (size_t)nb, hipMemcpyDeviceToHost, s->s_out));
        }
        APM_HIP(hipEventRecord(s->ev_d2h[slot], s->s_out));
    }
    APM_HIP(hipEventRecord(s->ev_done, s->s_out));
    APM_HIP(hipStreamWaitEvent(caller, s->ev_done, 0));
    return APM_OK;
}
}  // namespace

extern "C" int apm_streamer_step(apm_streamer* s, int64_t step, const apm_hyper* hyper,
                                 float* grad_norm, uint8_t* skip_mask, void* stream) {
    if (!s) return fail(APM_EINVAL, "NULL streamer");
    return run_pipeline(s, kDoH2D | kDoD2H | kDoUpdate, step, hyper, grad_norm, skip_mask, stream);
}

extern "C" int apm_streamer_set_cache(apm_streamer* s, apm_pool* cache, int64_t n_resident) {
    if (!s) return fail(APM_EINVAL, "NULL streamer");
    if (!cache || n_resident == 0) {
        s->cache = nullptr;
        s->R = 0;
        return APM_OK;
    }
    if (cache->desc.device != APM_DEV_GPU) return fail(APM_EDEVICE, "the cache must be a GPU pool");
    for (int st : {APM_P32, APM_M32, APM_V32}) if (!cache->stores(st)) return fail(APM_ESTATE, "cache pool lacks fp32 class %d", st);
    if (cache->desc.page_elems != s->dev->desc.page_elems) return fail(APM_EINVAL, "pools have different page sizes");
    if (n_resident < 0 || n_resident > cache->desc.n_pages) return fail(APM_ERANGE, "n_resident %lld exceeds the cache pool's %lld pages", (long long)n_resident, (long long)cache->desc.n_pages);
    s->cache = cache;
    s->R = n_resident;
    return APM_OK;
}

extern "C" int apm_streamer_copy_only(apm_streamer* s, int directions, void* stream) {
    if (!s) return fail(APM_EINVAL, "NULL streamer");
    if (directions < 1 || directions > 3) return fail(APM_EINVAL, "directions must be 1 (H2D), 2 (D2H) or 3 (both)");
    return run_pipeline(s, directions, 1, nullptr, nullptr, nullptr, stream);
}
