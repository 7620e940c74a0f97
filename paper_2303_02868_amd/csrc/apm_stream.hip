// Streamed update: fp32 master / momentum / variance pages live in pinned host memory
// (Sec. 4.2: overlap movement with computation; Sec. 5 "Allocator": asynchronous page copies; the
// update is page-granular by Sec. 4.3's last paragraph).  Two ways across PCIe:
//
// Staged mode: the pages pass through a small ring of HBM staging slots.  While batch b is updated
// in its slot on the compute stream, one copy kernel on the copy stream brings batch b+1 into the
// next slot and takes batch b-1 out of the previous one, both directions at once
// (apm_duplex_copy_kernel).  Staged-DMA mode is the same ring with the runtime's asynchronous
// copies instead: copy-in, update and copy-out each on its own stream.
//
// Mixed residency (Sec. 4.2, the GPU cache of optimizer states): the first R pages may keep their
// fp32 classes in a GPU pool; they are updated in place, in chunks interleaved with the streamed
// batches on the compute stream, and only pages [R, N) cross PCIe.
//
// Direct mode (apm_streamer_set_mode): no staging and no copies at all -- the update kernel reads
// p, m, v from the pinned host pages and writes them back across PCIe itself, with a small fixed
// number of wavefronts; the link carries both directions at once inside one kernel.
//
// Slot life cycle for batch b (slot = b mod n_slots), staged-DMA mode:
//   copy-in : wait D2H(b - n_slots) -> H2D p,m,v           -> record h2d[slot]
//   compute : wait h2d[slot]        -> reduce + update      -> record cmp[slot]
//   copy-out: wait cmp[slot]        -> D2H p,m,v            -> record d2h[slot]
// Streams are in order, so these three edges are the only synchronisation needed.  The host
// enqueues copy-in one batch ahead of the matching update and copy-out.
#include <algorithm>
#include <chrono>
#include <cstdlib>
#include <deque>

#include "apm_internal.h"

struct apm_streamer {
    apm_pool* host = nullptr;
    apm_pool* dev = nullptr;
    apm_pool* cache = nullptr;  // optional GPU pool holding the fp32 classes of pages [0, R)
    int64_t R = 0;              // number of leading pages whose fp32 state is HBM-resident
    int64_t host_first = 0;     // model page held by page 0 of the host pool
    int64_t page_limit = -1;    // the step covers model pages [0, page_limit); -1 = all pages in use
    int64_t B = 0;
    int n_slots = 0;
    float* stage[3] = {nullptr, nullptr, nullptr};  // each n_slots * B * E floats
    hipStream_t s_in = nullptr, s_cmp = nullptr, s_out = nullptr;
    bool host_wt = false;  // stores to the host pool written through at system scope (see apm.h)
    hipStream_t s_copy = nullptr;  // staged mode: the stream of the duplex copy kernels
    hipStream_t s_res = nullptr;  // direct mode: the resident pages' update, beside the host pages'
    hipEvent_t ev_res = nullptr;
    std::vector<hipEvent_t> ev_h2d, ev_cmp, ev_d2h;
    hipEvent_t ev_start = nullptr, ev_done = nullptr;
    bool in_is_null = false, out_is_null = false;  // a chosen copy stream may be the default stream
    double probe_h2d = 0, probe_d2h = 0, probe_duplex = 0;  // GB/s seen by the stream calibration
    int mode = APM_STREAM_STAGED;
    int direct_waves = 0;       // wavefronts of the direct-mode update kernel
    int direct_per_wg = 1;      // how many of them share a workgroup
    float* host_dev[3] = {nullptr, nullptr, nullptr};  // device-side addresses of the host pool's fp32 classes
    std::vector<hipEvent_t> sched_ev;  // events of the scheduled step, grown on demand and reused
    // one-step-stale form: the producer stream the pipeline's streams were last checked against
    bool paired = false;
    hipStream_t paired_with = nullptr;
    int paired_mode = -1;
    bool pair_overlaps = false;
};

using namespace apm;

namespace {
// Wavefronts of the direct-mode kernel when the caller names no number: kDirectWavefronts.
// Measured on MI355X (PCIe Gen5 x16, GB/s each way, 4 MiB pages, one wavefront per workgroup):
// 24 -> 44.5, 32 -> 46.6,
// 40 -> 48.4, 48 -> 49.5, 56 -> 49.4, 64 -> 49.0, 80 -> 48.3, 96 -> 48.0, 256 and more -> 45.4.
// Packed onto fewer CUs a CU's own memory pipeline becomes the limit: 64 wavefronts reach
// 47 GB/s at 8 per workgroup and 35 GB/s at 16; 128 at 16 reach 48.

void free_streamer(apm_streamer* s) {
    (void)hipDeviceSynchronize();
    if (s->s_in && !s->in_is_null) (void)hipStreamDestroy(s->s_in);
    if (s->s_out && !s->out_is_null) (void)hipStreamDestroy(s->s_out);
    if (s->s_cmp) (void)hipStreamDestroy(s->s_cmp);
    if (s->s_copy) (void)hipStreamDestroy(s->s_copy);
    if (s->s_res) (void)hipStreamDestroy(s->s_res);
    if (s->ev_res) (void)hipEventDestroy(s->ev_res);
    for (auto* v : {&s->ev_h2d, &s->ev_cmp, &s->ev_d2h, &s->sched_ev})
        for (hipEvent_t e : *v) if (e) (void)hipEventDestroy(e);
    if (s->ev_start) (void)hipEventDestroy(s->ev_start);
    if (s->ev_done) (void)hipEventDestroy(s->ev_done);
    for (float* p : s->stage) if (p) (void)hipFree(p);
    delete s;
}

// Which pairs of HIP streams run a host-to-device and a device-to-host copy at the same time is
// not something the API states: on the MI355X machine this was written on, a process has two groups of
// streams (the default stream and the first stream created form one, every later stream the
// other); copies on two streams of one group run one after the other (29 GB/s each way), copies on
// streams of different groups overlap (49 GB/s each way).  So the pair is chosen by measurement:
// a few candidate streams (the default stream among them) are timed on short concurrent copies
// through the staging memory, and the best pair becomes (copy-in, copy-out).
// beside (with use_beside): a stream whose work must not be held up by the pair -- the producer's,
// for the one-step-stale form.  Then the default stream is no candidate, and neither is a stream
// that shares a hardware queue with `beside` (measured with a pair of short kernels): an event
// wait enqueued on such a stream would hold up the kernels `beside` carries.
int pick_copy_streams(apm_streamer* s, hipStream_t beside = nullptr, bool use_beside = false) {
    constexpr int kNew = 5;
    constexpr size_t kProbe = (size_t)32 << 20;
    hipStream_t cand[kNew + 1] = {nullptr};  // cand[0] = the default stream
    bool usable[kNew + 1];
    for (int k = 1; k <= kNew; ++k) APM_HIP(hipStreamCreateWithFlags(&cand[k], hipStreamNonBlocking));
    for (int k = 0; k <= kNew; ++k) usable[k] = true;
    if (use_beside) {
        usable[0] = false;
        int n_ok = 0;
        bool ok[kNew + 1] = {false};
        for (int k = 1; k <= kNew; ++k) {
            int rc0 = streams_overlap(beside, cand[k], &ok[k]);
            if (rc0 != APM_OK) {
                for (int j = 1; j <= kNew; ++j) (void)hipStreamDestroy(cand[j]);
                return rc0;
            }
            n_ok += ok[k] ? 1 : 0;
        }
        if (n_ok >= 2)  // otherwise: nothing to choose from, keep them all
            for (int k = 1; k <= kNew; ++k) usable[k] = ok[k];
    }
    int first_ok = 0, second_ok = 0;
    for (int k = kNew; k >= 1; --k)
        if (usable[k]) { second_ok = first_ok; first_ok = k; }
    if (first_ok == 0 || second_ok == 0) { first_ok = 1; second_ok = 2; }
    char* h = nullptr;
    if (hipHostMalloc((void**)&h, 2 * kProbe, hipHostMallocDefault) != hipSuccess) {
        // no pinned memory left for the probe (the host pool may have taken it all): go without
        (void)hipGetLastError();
        s->s_in = cand[first_ok];
        s->s_out = cand[second_ok];
        s->in_is_null = s->out_is_null = false;
        for (int k = 1; k <= kNew; ++k)
            if (k != first_ok && k != second_ok) (void)hipStreamDestroy(cand[k]);
        return APM_OK;
    }
    const size_t slot_bytes = (size_t)s->B * (size_t)s->dev->desc.page_elems * sizeof(float);
    const size_t n = slot_bytes < kProbe ? slot_bytes : kProbe;
    char* d_in = reinterpret_cast<char*>(s->stage[0]);   // staging is not in use yet
    char* d_out = reinterpret_cast<char*>(s->stage[1]);
    auto timed = [&](hipStream_t a, hipStream_t b, bool do_in, bool do_out, double* gbps) -> int {
        APM_HIP(hipDeviceSynchronize());
        const auto t0 = std::chrono::steady_clock::now();
        for (int r = 0; r < 3; ++r) {
            if (do_in) APM_HIP(hipMemcpyAsync(d_in, h, n, hipMemcpyHostToDevice, a));
            if (do_out) APM_HIP(hipMemcpyAsync(h + kProbe, d_out, n, hipMemcpyDeviceToHost, b));
        }
        APM_HIP(hipDeviceSynchronize());
        const double dt = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
        *gbps = 3.0 * (double)n / dt / 1e9;
        return APM_OK;
    };
    double warm;
    int rc = timed(cand[first_ok], cand[second_ok], true, true, &warm);
    if (rc == APM_OK) rc = timed(cand[first_ok], cand[second_ok], true, false, &s->probe_h2d);
    if (rc == APM_OK) rc = timed(cand[first_ok], cand[second_ok], false, true, &s->probe_d2h);
    int bi = first_ok, bj = second_ok;
    double best = 0.0;
    for (int i = 0; i <= kNew && rc == APM_OK; ++i)
        for (int j = 0; j <= kNew && rc == APM_OK; ++j) {
            if (i == j || !usable[i] || !usable[j]) continue;
            double g;
            rc = timed(cand[i], cand[j], true, true, &g);
            if (rc == APM_OK && g > best) { best = g; bi = i; bj = j; }
        }
    (void)hipHostFree(h);
    if (rc != APM_OK) {
        for (int k = 1; k <= kNew; ++k) (void)hipStreamDestroy(cand[k]);
        return rc;
    }
    s->probe_duplex = best;
    s->s_in = cand[bi];
    s->s_out = cand[bj];
    s->in_is_null = bi == 0;
    s->out_is_null = bj == 0;
    for (int k = 1; k <= kNew; ++k)
        if (k != bi && k != bj) (void)hipStreamDestroy(cand[k]);
    return APM_OK;
}

int ensure_staging(apm_streamer* s);

// Staging slots, the copy streams and the per-slot events: set up when a staged mode is first
// asked for.  dma: the mode that uses the runtime's copies needs its calibrated stream pair; the
// kernel-copy mode needs one more stream only.
int ensure_staged(apm_streamer* s, bool dma) {
    APM_HIP(hipSetDevice(s->dev->desc.hip_device));
    int rc = ensure_staging(s);
    if (rc != APM_OK) return rc;
    if (dma && !s->s_in) return pick_copy_streams(s);
    if (!dma && !s->s_copy) {
        // The copy kernels must run beside the update kernels of the compute stream, which streams
        // that share a hardware queue do not: the copy stream is chosen by measurement.
        bool ok = false;
        return make_overlapping_stream(s->s_cmp, &s->s_copy, &ok);
    }
    return APM_OK;
}

int ensure_staging(apm_streamer* s) {
    if (s->stage[0]) return APM_OK;
    const size_t bytes = (size_t)s->n_slots * (size_t)s->B * (size_t)s->dev->desc.page_elems * sizeof(float);
    hipError_t e = hipSuccess;
    for (int k = 0; k < 3 && e == hipSuccess; ++k) e = hipMalloc((void**)&s->stage[k], bytes);
    auto undo = [&]() {
        for (float*& p : s->stage) {
            if (p) (void)hipFree(p);
            p = nullptr;
        }
    };
    if (e != hipSuccess) {
        (void)hipGetLastError();
        undo();
        return fail(APM_ENOMEM, "allocating 3 x %zu bytes of staging slots failed: %s", bytes, hipGetErrorString(e));
    }
    auto mk_event = [&](hipEvent_t* ev) { return *ev ? hipSuccess : hipEventCreateWithFlags(ev, hipEventDisableTiming); };
    s->ev_h2d.resize((size_t)s->n_slots, nullptr);
    s->ev_cmp.resize((size_t)s->n_slots, nullptr);
    s->ev_d2h.resize((size_t)s->n_slots, nullptr);
    for (int k = 0; k < s->n_slots && e == hipSuccess; ++k) {
        e = mk_event(&s->ev_h2d[(size_t)k]);
        if (e == hipSuccess) e = mk_event(&s->ev_cmp[(size_t)k]);
        if (e == hipSuccess) e = mk_event(&s->ev_d2h[(size_t)k]);
    }
    if (e != hipSuccess) {
        undo();
        return fail(APM_EDEVICE, "creating events failed: %s", hipGetErrorString(e));
    }
    return APM_OK;
}

// Device-side addresses of the host pool's fp32 classes (pinned memory is mapped into the GPU's
// address space); false if the memory cannot be addressed from the GPU.
bool map_host_classes(apm_streamer* s) {
    if (s->host_dev[0]) return true;
    const int states[3] = {APM_P32, APM_M32, APM_V32};
    float* p[3];
    for (int k = 0; k < 3; ++k) {
        if (hipHostGetDevicePointer((void**)&p[k], s->host->base[states[k]], 0) != hipSuccess) {
            (void)hipGetLastError();
            return false;
        }
    }
    for (int k = 0; k < 3; ++k) s->host_dev[k] = p[k];
    return true;
}

}  // namespace

extern "C" int apm_streamer_create(apm_streamer** out, apm_pool* host, apm_pool* dev,
                                   int64_t batch_pages, int n_slots) {
    return apm::guarded([&]() -> int {
        if (!out || !host || !dev) return fail(APM_EINVAL, "NULL argument");
        if (host->desc.device != APM_DEV_HOST || dev->desc.device != APM_DEV_GPU) return fail(APM_EDEVICE, "expected a HOST pool and a GPU pool");
        for (int st : {APM_P32, APM_M32, APM_V32}) if (!host->stores(st)) return fail(APM_ESTATE, "host pool lacks fp32 class %d", st);
        for (int st : {APM_G16, APM_P16}) if (!dev->stores(st)) return fail(APM_ESTATE, "GPU pool lacks 16-bit class %d", st);
        if (host->desc.page_elems != dev->desc.page_elems) return fail(APM_EINVAL, "pools have different page sizes");
        if (batch_pages < 1 || batch_pages > dev->desc.n_pages) return fail(APM_EINVAL, "batch_pages out of range");
        if (n_slots < 2 || n_slots > 64) return fail(APM_EINVAL, "n_slots must be in [2, 64]");
        APM_HIP(hipSetDevice(dev->desc.hip_device));
        apm_streamer* s = new apm_streamer();
        s->host = host; s->dev = dev; s->B = batch_pages; s->n_slots = n_slots;
        s->direct_waves = kDirectWavefronts;
        hipError_t e = hipStreamCreateWithFlags(&s->s_cmp, hipStreamNonBlocking);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&s->ev_start, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&s->ev_done, hipEventDisableTiming);
        if (e != hipSuccess) {
            free_streamer(s);
            return fail(APM_EDEVICE, "creating streams/events failed: %s", hipGetErrorString(e));
        }
        int rc = ensure_scratch(dev);
        if (rc == APM_OK) {
            if (map_host_classes(s)) s->mode = APM_STREAM_DIRECT;
            else { s->mode = APM_STREAM_STAGED_DMA; rc = ensure_staged(s, true); }
        }
        if (rc != APM_OK) { free_streamer(s); return rc; }
        *out = s;
        return APM_OK;
    });
}

extern "C" int apm_streamer_destroy(apm_streamer* s) {
    return apm::guarded([&]() -> int {
        if (!s) return APM_OK;
        (void)hipSetDevice(s->dev->desc.hip_device);
        free_streamer(s);
        return APM_OK;
    });
}

namespace {
enum { kDoH2D = 1, kDoD2H = 2, kDoUpdate = 4 };

// The pipeline.  `what` selects its parts: the full step uses all three; the copy-only
// measurement entry point drops the kernels (and optionally one direction) but keeps the streams,
// the event structure and the copy sizes.
int run_pipeline(apm_streamer* s, int what, int64_t step, const apm_hyper* hyper, float* grad_norm,
                 uint8_t* skip_mask, void* stream, const uint16_t* g16_override = nullptr) {
    apm_pool* dev = s->dev;
    apm_pool* host = s->host;
    if (!dev->has_layout) return fail(APM_ESTATE, "the GPU pool has no layout");
    AdamwLaunch L{};
    int rc = APM_OK;
    if (what & kDoUpdate) rc = prepare_hyper(hyper, step, &L);
    if (rc != APM_OK) return rc;
    APM_HIP(hipSetDevice(dev->desc.hip_device));
    hipStream_t caller = static_cast<hipStream_t>(stream);
    const int64_t in_use = (int64_t)dev->plan.pages.size();
    const int64_t N = s->page_limit >= 0 && s->page_limit < in_use ? s->page_limit : in_use;
    const int64_t E = dev->desc.page_elems;
    const size_t pb = (size_t)E * sizeof(float);

    const bool direct = s->mode == APM_STREAM_DIRECT;
    if (direct && !(what & kDoUpdate)) return fail(APM_ESTATE, "the copy-only measurement belongs to the staged modes; this streamer is in direct mode");
    APM_HIP(hipEventRecord(s->ev_start, caller));
    APM_HIP(hipStreamWaitEvent(s->s_cmp, s->ev_start, 0));
    const bool kcopy = s->mode == APM_STREAM_STAGED;
    if (kcopy) {
        APM_HIP(hipStreamWaitEvent(s->s_copy, s->ev_start, 0));
    } else if (!direct) {
        APM_HIP(hipStreamWaitEvent(s->s_in, s->ev_start, 0));
        APM_HIP(hipStreamWaitEvent(s->s_out, s->ev_start, 0));
    }

    L.g16 = g16_override ? g16_override : static_cast<const uint16_t*>(dev->base[APM_G16]);
    L.p16 = static_cast<uint16_t*>(dev->base[APM_P16]);
    L.used = dev->d_used;
    L.E = E;
    L.S = dev->S;
    L.p32 = s->stage[0];
    L.m32 = s->stage[1];
    L.v32 = s->stage[2];
    const bool need_reduce = grad_norm || skip_mask || L.max_norm > 0.0 || L.skip_mode != APM_SKIP_NONE;
    L.meta = dev->d_meta;
    if (need_reduce) {
        L.partials = dev->d_partials;
        L.nzflags = dev->d_nzflags;
    }
    const int states[3] = {APM_P32, APM_M32, APM_V32};
    const int64_t R = s->cache ? (s->R < N ? s->R : N) : 0;
    // host pool page j holds model page host_first + j; the pages before it must be resident
    const int64_t H0 = s->host_first;
    if (R < H0 && N > 0) return fail(APM_ESTATE, "model pages [%lld, %lld) are neither resident in the cache nor held by the host pool", (long long)R, (long long)H0);
    if (N - H0 > host->desc.n_pages) return fail(APM_ESTATE, "the host pool holds %lld pages, %lld are needed from model page %lld on", (long long)host->desc.n_pages, (long long)(N - H0), (long long)H0);
    if (direct) {
        // The resident pages (HBM speed) and the host pages (PCIe speed) are updated side by side
        // on two streams; each part has its own range of the per-page scratch.
        const bool two = R > 0 && R < N;
        if (two && !s->s_res) {  // a stream whose kernels run beside the compute stream's (measured)
            bool ok = false;
            rc = make_overlapping_stream(s->s_cmp, &s->s_res, &ok);
            if (rc != APM_OK) return rc;
            APM_HIP(hipEventCreateWithFlags(&s->ev_res, hipEventDisableTiming));
        }
        if (two) APM_HIP(hipStreamWaitEvent(s->s_res, s->ev_start, 0));
        for (int part = 0; part < 2; ++part) {
            AdamwLaunch C = L;
            const int64_t first = part == 0 ? 0 : R;
            const int64_t n = part == 0 ? R : N - R;
            if (n == 0) continue;
            hipStream_t st = part == 0 && two ? s->s_res : s->s_cmp;
            if (part == 0) {
                C.p32 = static_cast<float*>(s->cache->base[APM_P32]);
                C.m32 = static_cast<float*>(s->cache->base[APM_M32]);
                C.v32 = static_cast<float*>(s->cache->base[APM_V32]);
            } else {
                C.p32 = s->host_dev[0];
                C.m32 = s->host_dev[1];
                C.v32 = s->host_dev[2];
                C.stride_wavefronts = s->direct_waves;
                C.stride_waves_per_wg = s->direct_per_wg;
                C.host_write_through = s->host_wt;
            }
            C.meta = L.meta + first;
            if (need_reduce) {
                C.partials = L.partials + first * L.S;
                C.nzflags = L.nzflags + first * L.S;
            }
            C.state_first = part == 0 ? first : first - H0;
            C.grad_first = first;
            C.n_listed = n;
            C.grad_norm = grad_norm ? grad_norm + first : nullptr;
            C.skip_mask = skip_mask ? skip_mask + first : nullptr;
            if (need_reduce) APM_HIP(launch_grad_reduce(C, st));
            else APM_HIP(launch_prepare(C, st));
            APM_HIP(launch_adamw(C, st));
        }
        if (two) {
            APM_HIP(hipEventRecord(s->ev_res, s->s_res));
            APM_HIP(hipStreamWaitEvent(s->s_cmp, s->ev_res, 0));
        }
        APM_HIP(hipEventRecord(s->ev_done, s->s_cmp));
        APM_HIP(hipStreamWaitEvent(caller, s->ev_done, 0));
        return APM_OK;
    }
    // Batches: runs of at most B consecutive pages from page R on.  The runtime's copies move
    // whole pages, so there every batch has B pages.  The copy kernel moves used extents, and an
    // exchange takes as long as its longer direction, so there the batches are cut to hold about
    // the same number of used elements each: as many as the emptiest window of B pages holds (a
    // GPT layout has a nearly empty page in every seven or eight; with B pages per batch the two
    // directions of an exchange differed by 7 % on average, and the step was that much longer).
    std::vector<int64_t> batch_at;  // first page of batch b; one entry more than there are batches
    batch_at.push_back(R);
    if (kcopy && N - R > s->B) {
        const auto used_of = [&](int64_t p) { return (int64_t)dev->plan.pages[(size_t)p].used; };
        int64_t window = 0, emptiest = INT64_MAX;
        for (int64_t p = R; p < N; ++p) {
            window += used_of(p);
            if (p - R >= s->B) window -= used_of(p - s->B);
            if (p - R >= s->B - 1 && window < emptiest) emptiest = window;
        }
        int64_t in_batch = 0;
        for (int64_t p = R; p < N; ++p) {
            const int64_t u = used_of(p), n_here = p - batch_at.back();
            if (n_here > 0 && (n_here == s->B || in_batch + u / 2 > emptiest)) {  // nearest to the target
                batch_at.push_back(p);
                in_batch = 0;
            }
            in_batch += u;
        }
        batch_at.push_back(N);
    } else {
        for (int64_t p = R + s->B; p < N; p += s->B) batch_at.push_back(p);
        if (N > R) batch_at.push_back(N);
    }
    const int64_t n_batches = (int64_t)batch_at.size() - 1;
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
        else APM_HIP(launch_prepare(C, s->s_cmp));
        APM_HIP(launch_adamw(C, s->s_cmp));
        r_done += nr;
        return APM_OK;
    };
    hipStream_t s_last = kcopy ? s->s_copy : s->s_out;  // the stream the step ends on
    if (n_batches == 0) {
        rc = resident_chunk();
        if (rc != APM_OK) return rc;
        APM_HIP(hipEventRecord(s->ev_cmp[0], s->s_cmp));
        APM_HIP(hipStreamWaitEvent(s_last, s->ev_cmp[0], 0));
    }
    auto update_batch = [&](int64_t b) -> int {
        const size_t slot = (size_t)(b % s->n_slots);
        const int64_t first = batch_at[(size_t)b];
        const int64_t nb = batch_at[(size_t)b + 1] - first;
        APM_HIP(hipStreamWaitEvent(s->s_cmp, s->ev_h2d[slot], 0));
        L.state_first = (int64_t)slot * s->B;
        L.grad_first = first;
        L.n_listed = nb;
        L.grad_norm = grad_norm ? grad_norm + first : nullptr;
        L.skip_mask = skip_mask ? skip_mask + first : nullptr;
        if (what & kDoUpdate) {
            if (need_reduce) APM_HIP(launch_grad_reduce(L, s->s_cmp));
            else APM_HIP(launch_prepare(L, s->s_cmp));
            APM_HIP(launch_adamw(L, s->s_cmp));
        }
        APM_HIP(hipEventRecord(s->ev_cmp[slot], s->s_cmp));
        return APM_OK;
    };
    if (kcopy) {
        // Iteration b: one copy kernel brings batch b+1 in and takes batch b-1 out while batch b is
        // updated.  With three or more slots the three batches sit in different slots; with two,
        // the incoming batch reuses the outgoing batch's slot, so the two directions become two
        // kernels, one after the other.
        auto exchange = [&](int64_t b_in, int64_t b_out) -> int {
            DuplexCopy d{};
            auto fill = [&](int64_t b, bool in) {
                const size_t slot = (size_t)(b % s->n_slots);
                const int64_t first = batch_at[(size_t)b];
                const int64_t nb = batch_at[(size_t)b + 1] - first;
                const size_t slot_off = slot * (size_t)s->B * (size_t)E;  // floats
                for (int k = 0; k < 3; ++k) {
                    char* h = reinterpret_cast<char*>(s->host_dev[k]) + (size_t)(first - H0) * pb;
                    char* g = reinterpret_cast<char*>(s->stage[k] + slot_off);
                    if (in) { d.in_src[k] = h; d.in_dst[k] = g; }
                    else { d.out_src[k] = g; d.out_dst[k] = h; }
                }
                (in ? d.in_bytes : d.out_bytes) = (int64_t)(pb * (size_t)nb);
                (in ? d.in_first_page : d.out_first_page) = first;
            };
            d.used = dev->d_used;  // only the used extents cross the link
            d.page_bytes = (int64_t)pb;
            d.host_store_policy = s->host_wt ? 3 : 0;
            if (b_in >= 0 && (what & kDoH2D)) fill(b_in, true);
            if (b_out >= 0 && (what & kDoD2H)) fill(b_out, false);
            APM_HIP(launch_duplex_copy(d, s->direct_waves, s->direct_per_wg, s->s_copy));
            return APM_OK;
        };
        if (n_batches > 0) {
            rc = exchange(0, -1);
            if (rc != APM_OK) return rc;
            APM_HIP(hipEventRecord(s->ev_h2d[0], s->s_copy));
        }
        for (int64_t b = 0; b < n_batches; ++b) {
            const bool has_in = b + 1 < n_batches, has_out = b >= 1;
            if (has_out) APM_HIP(hipStreamWaitEvent(s->s_copy, s->ev_cmp[(size_t)((b - 1) % s->n_slots)], 0));
            if (has_in && has_out && s->n_slots < 3) {
                rc = exchange(-1, b - 1);
                if (rc == APM_OK) rc = exchange(b + 1, -1);
            } else if (has_in || has_out) {
                rc = exchange(has_in ? b + 1 : -1, has_out ? b - 1 : -1);
            }
            if (rc != APM_OK) return rc;
            if (has_in) APM_HIP(hipEventRecord(s->ev_h2d[(size_t)((b + 1) % s->n_slots)], s->s_copy));
            rc = resident_chunk();  // runs while this batch's neighbours are in flight
            if (rc == APM_OK) rc = update_batch(b);
            if (rc != APM_OK) return rc;
        }
        if (n_batches > 0) {
            APM_HIP(hipStreamWaitEvent(s->s_copy, s->ev_cmp[(size_t)((n_batches - 1) % s->n_slots)], 0));
            rc = exchange(-1, n_batches - 1);
            if (rc != APM_OK) return rc;
        }
        APM_HIP(hipEventRecord(s->ev_done, s->s_copy));
        APM_HIP(hipStreamWaitEvent(caller, s->ev_done, 0));
        return APM_OK;
    }
    // Copy-in is enqueued one batch ahead of the update that consumes it: when this was written the
    // runtime's device-to-host copy was a kernel whose enqueue blocked the host until the event it
    // waits for had fired, and without the look-ahead the copy-in stream idled during each update.  (A
    // look-ahead of two batches was measured to make the runtime run the two copy directions one
    // after the other, 28 instead of 48 GB/s each way, so one it is.)
    auto copy_in = [&](int64_t b) -> int {
        const size_t slot = (size_t)(b % s->n_slots);
        const int64_t first = batch_at[(size_t)b];
        const int64_t nb = batch_at[(size_t)b + 1] - first;
        const size_t slot_off = slot * (size_t)s->B * (size_t)E;  // floats
        if (b >= s->n_slots) APM_HIP(hipStreamWaitEvent(s->s_in, s->ev_d2h[slot], 0));
        for (int k = 0; k < 3 && (what & kDoH2D); ++k) {
            const char* src = static_cast<const char*>(host->base[states[k]]) + (size_t)(first - H0) * pb;
            APM_HIP(hipMemcpyAsync(s->stage[k] + slot_off, src, pb * (size_t)nb, hipMemcpyHostToDevice, s->s_in));
        }
        APM_HIP(hipEventRecord(s->ev_h2d[slot], s->s_in));
        return APM_OK;
    };
    const int64_t ahead = 1;
    for (int64_t b = 0; b < ahead && b < n_batches; ++b) {
        rc = copy_in(b);
        if (rc != APM_OK) return rc;
    }
    for (int64_t b = 0; b < n_batches; ++b) {
        const size_t slot = (size_t)(b % s->n_slots);
        const int64_t first = batch_at[(size_t)b];
        const int64_t nb = batch_at[(size_t)b + 1] - first;
        const size_t slot_off = slot * (size_t)s->B * (size_t)E;  // floats
        if (b + ahead < n_batches) {  // its slot's previous copy-out is already enqueued
            rc = copy_in(b + ahead);
            if (rc != APM_OK) return rc;
        }

        rc = resident_chunk();  // runs while this batch's copy-in is in flight
        if (rc == APM_OK) rc = update_batch(b);
        if (rc != APM_OK) return rc;

        APM_HIP(hipStreamWaitEvent(s->s_out, s->ev_cmp[slot], 0));
        for (int k = 0; k < 3 && (what & kDoD2H); ++k) {
            char* dst = static_cast<char*>(host->base[states[k]]) + (size_t)(first - H0) * pb;
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
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        return run_pipeline(s, kDoH2D | kDoD2H | kDoUpdate, step, hyper, grad_norm, skip_mask, stream);
    });
}

namespace {
// The one-step-stale form pays only if the pipeline's kernels run beside the producer's.  Streams
// that the runtime put on the producer stream's hardware queue are replaced (checked once per
// producer stream and mode; the streams must be idle, which they are between steps).
int pair_with_producer(apm_streamer* s, hipStream_t producer) {
    if (s->paired && s->paired_with == producer && s->paired_mode == s->mode) return APM_OK;
    APM_HIP(hipDeviceSynchronize());
    bool all = true;
    if (s->mode == APM_STREAM_STAGED_DMA && s->s_in) {
        // the calibrated pair may contain the default stream or share a hardware queue with the
        // producer's stream: pick it again among streams that stay clear of the producer
        if (!s->in_is_null) (void)hipStreamDestroy(s->s_in);
        if (!s->out_is_null) (void)hipStreamDestroy(s->s_out);
        s->s_in = s->s_out = nullptr;
        s->in_is_null = s->out_is_null = false;
        int rc = pick_copy_streams(s, producer, true);
        if (rc != APM_OK) return rc;
        bool a = false, b = false;
        rc = streams_overlap(producer, s->s_in, &a);
        if (rc == APM_OK) rc = streams_overlap(producer, s->s_out, &b);
        if (rc != APM_OK) return rc;
        all = a && b;
    }
    hipStream_t* pipeline[2] = {&s->s_cmp, s->mode == APM_STREAM_STAGED ? &s->s_copy : nullptr};
    for (hipStream_t* st : pipeline) {
        if (!st || !*st) continue;
        bool ok = false;
        int rc = streams_overlap(producer, *st, &ok);
        if (rc != APM_OK) return rc;
        if (!ok) {
            hipStream_t fresh = nullptr;
            rc = make_overlapping_stream(producer, &fresh, &ok);
            if (rc != APM_OK) return rc;
            (void)hipStreamDestroy(*st);
            *st = fresh;
        }
        all = all && ok;
    }
    s->paired = true;
    s->paired_with = producer;
    s->paired_mode = s->mode;
    s->pair_overlaps = all;
    return APM_OK;
}
}  // namespace

// Alg. 2 with the optimizer states off the GPU: the updating side is the streamed step (in direct
// mode a few dozen wavefronts working through the host pages), the buffering side the caller's
// stream handing over the next gradient.
extern "C" int apm_streamer_step_delayed(apm_streamer* s, const void* new_g16, const apm_hyper* hyper,
                                         void* stream) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        apm_pool* dev = s->dev;
        if (!dev->has_layout) return fail(APM_ESTATE, "the GPU pool has no layout");
        AdamwLaunch probe{};
        int rc = prepare_hyper(hyper, 1, &probe);  // validate before any state changes
        if (rc != APM_OK) return rc;
        const int64_t N = (int64_t)dev->plan.pages.size();
        if (s->mode != APM_STREAM_STAGED_DMA) {  // the runtime's copy queues are not ours to place
            APM_HIP(hipSetDevice(dev->desc.hip_device));
            rc = pair_with_producer(s, static_cast<hipStream_t>(stream));
            if (rc != APM_OK) return rc;
        }
        return delayed_call(dev, nullptr, N, new_g16, hyper, static_cast<hipStream_t>(stream),
                            [&](const uint16_t* g16, int64_t step, hipStream_t upd, const int64_t*, int64_t,
                                const apm_hyper* b_hyper) {
                                return run_pipeline(s, kDoH2D | kDoD2H | kDoUpdate, step, b_hyper, dev->delayed_norm,
                                                    dev->delayed_skip, upd, g16);
                            });
    });
}

extern "C" int apm_streamer_overlap_report(const apm_streamer* s, int* update_stream, int* pipeline_streams) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        if (update_stream) *update_stream = s->dev->upd_stream ? (s->dev->upd_overlaps ? 1 : 0) : -1;
        if (pipeline_streams) *pipeline_streams = s->paired ? (s->pair_overlaps ? 1 : 0) : -1;
        return APM_OK;
    });
}

extern "C" int apm_streamer_set_mode(apm_streamer* s, int mode, int direct_wavefronts,
                                     int wavefronts_per_workgroup) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        if (mode != APM_STREAM_STAGED && mode != APM_STREAM_DIRECT && mode != APM_STREAM_STAGED_DMA) return fail(APM_EINVAL, "unknown streamer mode %d", mode);
        if (direct_wavefronts < 0 || direct_wavefronts > (1 << 20)) return fail(APM_EINVAL, "direct_wavefronts out of range");
        if (wavefronts_per_workgroup < 0 || wavefronts_per_workgroup > 16) return fail(APM_EINVAL, "wavefronts_per_workgroup must be in [0, 16]");
        APM_HIP(hipSetDevice(s->dev->desc.hip_device));
        if (mode == APM_STREAM_DIRECT || mode == APM_STREAM_STAGED) {
            if (!map_host_classes(s)) return fail(APM_EDEVICE, "the host pool's memory is not mapped into the GPU's address space (not pinned?): only APM_STREAM_STAGED_DMA can serve it");
            s->direct_waves = direct_wavefronts > 0 ? direct_wavefronts : kDirectWavefronts;
            s->direct_per_wg = wavefronts_per_workgroup > 0 ? wavefronts_per_workgroup : 1;
        }
        if (mode != APM_STREAM_DIRECT) {
            int rc = ensure_staged(s, mode == APM_STREAM_STAGED_DMA);
            if (rc != APM_OK) return rc;
        }
        s->mode = mode;
        return APM_OK;
    });
}

extern "C" int apm_streamer_get_mode(const apm_streamer* s) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        return s->mode;
    });
}

extern "C" int apm_streamer_probe_rates(const apm_streamer* s, double* h2d, double* d2h, double* duplex_each_way) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        if (h2d) *h2d = s->probe_h2d;
        if (d2h) *d2h = s->probe_d2h;
        if (duplex_each_way) *duplex_each_way = s->probe_duplex;
        return APM_OK;
    });
}

extern "C" int apm_streamer_set_cache(apm_streamer* s, apm_pool* cache, int64_t n_resident) {
    return apm::guarded([&]() -> int {
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
    });
}

extern "C" int apm_cache_pages_that_fit(int hip_device, int64_t page_elems, int64_t n_pages,
                                        size_t reserve_bytes, int64_t* out) {
    return apm::guarded([&]() -> int {
        if (!out || page_elems <= 0 || n_pages < 0) return fail(APM_EINVAL, "bad argument");
        APM_HIP(hipSetDevice(hip_device));
        size_t free_b = 0, total_b = 0;
        APM_HIP(hipMemGetInfo(&free_b, &total_b));
        const size_t page_bytes = (size_t)page_elems * 3u * sizeof(float);
        const size_t usable = free_b > reserve_bytes ? free_b - reserve_bytes : 0;
        const int64_t fit = (int64_t)(usable / page_bytes);
        *out = fit < n_pages ? fit : n_pages;
        return APM_OK;
    });
}

extern "C" int apm_streamer_set_page_count(apm_streamer* s, int64_t n_pages) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        s->page_limit = n_pages < 0 ? -1 : n_pages;
        return APM_OK;
    });
}

extern "C" int apm_streamer_set_host_write_through(apm_streamer* s, int on) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        s->host_wt = on != 0;
        return APM_OK;
    });
}

extern "C" int apm_streamer_set_host_first_page(apm_streamer* s, int64_t first_model_page) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        if (first_model_page < 0 || first_model_page > s->dev->desc.n_pages) return fail(APM_ERANGE, "first_model_page out of range");
        s->host_first = first_model_page;
        return APM_OK;
    });
}

// One step driven by a schedule (Alg. 1's task list) instead of the fixed slot ring.  The staging
// memory is the GPU memory the schedule was planned for, one page slot per page; a movement task
// takes the lowest free slot, a compute task updates its layer's pages where they sit, writes them
// back and frees their slots.  The whole schedule is checked on the host before anything is
// enqueued.  Edges: a copy-in waits for its trigger and for the write-back that freed its slots, a
// compute for the copy-ins of its pages, a write-back for its compute.
extern "C" int apm_streamer_step_scheduled(apm_streamer* s, const apm_task* tasks, int64_t n_tasks,
                                           const int64_t* layer_first_page, int64_t n_layers,
                                           const int64_t* last_access, int64_t step,
                                           const apm_hyper* hyper, float* grad_norm,
                                           uint8_t* skip_mask, void* stream) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        if (n_tasks < 0 || n_layers < 0 || (n_tasks > 0 && !tasks) || !layer_first_page) return fail(APM_EINVAL, "bad task or layer arrays");
        apm_pool* dev = s->dev;
        apm_pool* host = s->host;
        if (!dev->has_layout) return fail(APM_ESTATE, "the GPU pool has no layout");
        const int64_t N = (int64_t)dev->plan.pages.size();
        if (layer_first_page[0] != 0 || layer_first_page[n_layers] != N) return fail(APM_EINVAL, "the layers must cover pages [0, %lld) in order", (long long)N);
        for (int64_t i = 0; i < n_layers; ++i)
            if (layer_first_page[i + 1] < layer_first_page[i]) return fail(APM_EINVAL, "layer_first_page must not decrease");
        if (s->cache || s->host_first != 0 || s->page_limit >= 0) return fail(APM_ESTATE, "the scheduled step does not combine with a resident cache or a page range");
        if (s->host->desc.n_pages < N) return fail(APM_ESTATE, "the host pool holds fewer pages than are in use");
        AdamwLaunch L{};
        int rc = prepare_hyper(hyper, step, &L);
        if (rc != APM_OK) return rc;
        APM_HIP(hipSetDevice(dev->desc.hip_device));
        // The page movement is the library's copy kernel unless the streamer is in staged-DMA mode or
        // the GPU cannot address the host pool; then it is the runtime's copies.
        const bool kcopy = s->mode != APM_STREAM_STAGED_DMA && map_host_classes(s);
        rc = ensure_staged(s, !kcopy);
        if (rc != APM_OK) return rc;
        hipStream_t s_in = kcopy ? s->s_copy : s->s_in, s_out = kcopy ? s->s_copy : s->s_out;

        // The trace: the layer after whose compute a page's slot is free again (its own layer if
        // no trace is given).  release_at[i] lists, in ascending order, the pages layer i releases.
        std::vector<int64_t> own((size_t)N, 0);
        for (int64_t i = 0; i < n_layers; ++i)
            for (int64_t p = layer_first_page[i]; p < layer_first_page[i + 1]; ++p) own[(size_t)p] = i;
        std::vector<std::vector<int64_t>> release_at((size_t)n_layers);
        for (int64_t p = 0; p < N; ++p) {
            const int64_t la = last_access ? last_access[p] : own[(size_t)p];
            if (la < own[(size_t)p] || la >= n_layers) return fail(APM_EINVAL, "last_access[%lld] = %lld lies outside [its own layer %lld, %lld)", (long long)p, (long long)la, (long long)own[(size_t)p], (long long)n_layers);
            release_at[(size_t)la].push_back(p);
        }

        // ---- pass 1 (host only): replay the schedule against the slots -------------------------
        const int64_t n_slots = (int64_t)s->n_slots * s->B;
        std::vector<int64_t> slot_of((size_t)N, -1);
        std::vector<uint8_t> moved((size_t)N, 0);
        std::vector<int64_t> free_slots((size_t)n_slots);  // min-heap: the lowest free slot first keeps runs together
        for (int64_t k = 0; k < n_slots; ++k) free_slots[(size_t)k] = k;
        auto cmp = [](int64_t a, int64_t b) { return a > b; };
        std::make_heap(free_slots.begin(), free_slots.end(), cmp);
        std::vector<int64_t> slot_seq((size_t)N, -1);  // slot given to each movement task, by page
        int64_t next_layer = 0, n_moves = 0;
        for (int64_t k = 0; k < n_tasks; ++k) {
            const apm_task& t = tasks[k];
            if (t.op == APM_TASK_MOVE_TO_GPU) {
                if (t.target < 0 || t.target >= N) return fail(APM_ERANGE, "task %lld moves page %lld, out of range", (long long)k, (long long)t.target);
                if (moved[(size_t)t.target]) return fail(APM_EINVAL, "task %lld moves page %lld a second time", (long long)k, (long long)t.target);
                // A movement is issued when execution reaches its trigger id, i.e. once the layer
                // before it has computed.  A trigger beyond the layers that precede the task in the
                // list could never fire before the computes that wait for this very page.
                if (t.trigger_id < 0 || t.trigger_id > next_layer) return fail(APM_EINVAL, "task %lld: trigger id %d is not in [0, %lld], the layers whose turn has come at this point of the list", (long long)k, t.trigger_id, (long long)next_layer);
                if (free_slots.empty()) return fail(APM_ENOMEM, "task %lld: the schedule needs more than the %lld staging page slots", (long long)k, (long long)n_slots);
                std::pop_heap(free_slots.begin(), free_slots.end(), cmp);
                slot_seq[(size_t)t.target] = slot_of[(size_t)t.target] = free_slots.back();
                free_slots.pop_back();
                moved[(size_t)t.target] = 1;
                ++n_moves;
            } else if (t.op == APM_TASK_COMPUTE) {
                if (t.target != next_layer) return fail(APM_EINVAL, "task %lld computes layer %lld, expected layer %lld", (long long)k, (long long)t.target, (long long)next_layer);
                for (int64_t p = layer_first_page[next_layer]; p < layer_first_page[next_layer + 1]; ++p)
                    if (slot_of[(size_t)p] < 0) return fail(APM_ESTATE, "task %lld computes layer %lld before its page %lld was moved", (long long)k, (long long)next_layer, (long long)p);
                for (int64_t p : release_at[(size_t)next_layer]) {  // moved: its own layer has computed
                    free_slots.push_back(slot_of[(size_t)p]);
                    std::push_heap(free_slots.begin(), free_slots.end(), cmp);
                    slot_of[(size_t)p] = -1;
                }
                ++next_layer;
            } else {
                return fail(APM_EINVAL, "task %lld has unknown operation %d", (long long)k, t.op);
            }
        }
        if (next_layer != n_layers || n_moves != N) return fail(APM_EINVAL, "the schedule computes %lld of %lld layers and moves %lld of %lld pages", (long long)next_layer, (long long)n_layers, (long long)n_moves, (long long)N);

        // ---- pass 2: enqueue --------------------------------------------------------------------
        hipStream_t caller = static_cast<hipStream_t>(stream);
        const int64_t E = dev->desc.page_elems;
        const size_t pb = (size_t)E * sizeof(float);
        const int states[3] = {APM_P32, APM_M32, APM_V32};
        size_t ev_used = 0;
        auto new_event = [&](hipEvent_t* out) -> int {
            if (ev_used == s->sched_ev.size()) {
                hipEvent_t e = nullptr;
                APM_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
                s->sched_ev.push_back(e);
            }
            *out = s->sched_ev[ev_used++];
            return APM_OK;
        };
        APM_HIP(hipEventRecord(s->ev_start, caller));
        APM_HIP(hipStreamWaitEvent(s_in, s->ev_start, 0));
        APM_HIP(hipStreamWaitEvent(s->s_cmp, s->ev_start, 0));
        APM_HIP(hipStreamWaitEvent(s_out, s->ev_start, 0));

        // the slot of every page, for the kernels (fp32 classes are addressed by slot, 16-bit ones by page)
        int slots_ring_slot = -1;
        {
            int slot;
            rc = dev->ring.acquire((size_t)N * sizeof(int64_t), &slot);
            if (rc != APM_OK) return rc;
            int64_t* h = static_cast<int64_t*>(dev->ring.h[slot]);
            for (int64_t p = 0; p < N; ++p) h[p] = slot_seq[(size_t)p];
            rc = dev->ring.commit(slot, (size_t)N * sizeof(int64_t), s->s_cmp);
            if (rc != APM_OK) return rc;
            slots_ring_slot = slot;
            L.state_pages = static_cast<const int64_t*>(dev->ring.d[slot]);
        }
        L.g16 = static_cast<const uint16_t*>(dev->base[APM_G16]);
        L.p16 = static_cast<uint16_t*>(dev->base[APM_P16]);
        L.used = dev->d_used;
        L.E = E;
        L.S = dev->S;
        L.p32 = s->stage[0];
        L.m32 = s->stage[1];
        L.v32 = s->stage[2];
        L.meta = dev->d_meta;
        const bool need_reduce = grad_norm || skip_mask || L.max_norm > 0.0 || L.skip_mode != APM_SKIP_NONE;
        if (need_reduce) {
            L.partials = dev->d_partials;
            L.nzflags = dev->d_nzflags;
        }
        const int64_t* d_slots = L.state_pages;

        std::vector<hipEvent_t> slot_free((size_t)n_slots, nullptr);  // write-back that last freed the slot
        std::vector<hipEvent_t> page_in((size_t)N, nullptr);          // copy-in that brought the page
        // reached[t]: logical time t, the point of the compute stream where layer t - 1 has
        // computed (t = 0: the start of the step).  A movement task waits for reached[trigger_id]
        // (event-driven dispatch, Sec. 5 "Unified Scheduler") besides the slots it moves into.
        std::vector<hipEvent_t> reached((size_t)n_layers + 1, nullptr);
        hipEvent_t last_computed = nullptr;
        // reduce + update of pages [first, first + n) on the compute stream, once they have arrived
        auto compute_pages = [&](int64_t first, int64_t n, hipEvent_t* computed) -> int {
            if (n > 0) {
                hipEvent_t last_wait = nullptr;
                for (int64_t j = 0; j < n; ++j) {
                    hipEvent_t w = page_in[(size_t)(first + j)];
                    if (w != last_wait) {
                        APM_HIP(hipStreamWaitEvent(s->s_cmp, w, 0));
                        last_wait = w;
                    }
                }
                AdamwLaunch C = L;
                C.state_pages = d_slots + first;
                C.grad_first = first;
                C.n_listed = n;
                C.grad_norm = grad_norm ? grad_norm + first : nullptr;
                C.skip_mask = skip_mask ? skip_mask + first : nullptr;
                if (need_reduce) APM_HIP(launch_grad_reduce(C, s->s_cmp));
                else APM_HIP(launch_prepare(C, s->s_cmp));
                APM_HIP(launch_adamw(C, s->s_cmp));
            }
            int rc2 = new_event(computed);
            if (rc2 != APM_OK) return rc2;
            APM_HIP(hipEventRecord(*computed, s->s_cmp));
            last_computed = *computed;
            return APM_OK;
        };
        // one layer's compute; records logical time i + 1, which is also what the write-back of the
        // pages released here waits for
        auto compute_layer = [&](int64_t i, hipEvent_t* computed) -> int {
            int rc2 = compute_pages(layer_first_page[i], layer_first_page[i + 1] - layer_first_page[i], computed);
            if (rc2 == APM_OK) reached[(size_t)i + 1] = *computed;
            return rc2;
        };

        if (kcopy) {
            // One copy stream, and one kernel per exchange: the write-back of the pages a layer
            // releases travels together with movement tasks that are due, so that the link carries
            // both directions inside one kernel (two kernels, one per direction, reach four fifths
            // of that).  A movement task is never issued before its trigger id is reached, but it
            // may be issued later: it is held back until a write-back can take it along, two layers
            // ahead of the compute that needs its page (one layer ahead would put every compute
            // between two copy kernels), or, at the latest, right before that compute.  Slots need
            // no events here: the write-back that frees a slot precedes, in this one stream, the
            // movement that reuses it, because it precedes it in the task list.
            //
            // The optimizer's pages are independent, so a layer's compute task is carried out in
            // units of at most kUnit pages, each written back as soon as it has computed: the
            // first layer (the embedding, a seventh of a GPT-shaped model's pages) then need not
            // arrive whole before anything flows back, nor the last one leave alone at the end.
            // Slots are freed no later than the schedule says, and movements keep their place in
            // the list, so the replay above still covers what is enqueued here.
            constexpr int64_t kUnit = 16;  // measured on the 1.3 B shape: 8 / 16 / 32 pages -> 351 / 341 / 363 ms per step
            std::vector<int64_t> unit_first;                       // first page of unit u (+ one end entry)
            std::vector<int64_t> first_unit((size_t)n_layers + 1);  // layer i's first unit
            for (int64_t i = 0; i < n_layers; ++i) {
                first_unit[(size_t)i] = (int64_t)unit_first.size();
                int64_t q = layer_first_page[i];
                do {  // a layer without pages is one empty unit
                    unit_first.push_back(q);
                    q += kUnit;
                } while (q < layer_first_page[i + 1]);
            }
            const int64_t n_units = (int64_t)unit_first.size();
            first_unit[(size_t)n_layers] = n_units;
            unit_first.push_back(N);
            // what unit u releases: its own pages whose last access is their own layer, and, for a
            // layer's last unit, the pages of earlier layers that the trace kept until this layer
            std::vector<std::vector<int64_t>> unit_release((size_t)n_units);
            for (int64_t i = 0; i < n_layers; ++i)
                for (int64_t q : release_at[(size_t)i]) {
                    int64_t u = first_unit[(size_t)i + 1] - 1;
                    if (own[(size_t)q] == i) u = first_unit[(size_t)i] + (q - layer_first_page[i]) / kUnit;
                    unit_release[(size_t)u].push_back(q);
                }
            for (auto& v : unit_release) std::sort(v.begin(), v.end());
            // logical time in units: reached_u[u] = unit u - 1 has computed; trigger id t (a layer)
            // is reached when the last unit of layer t - 1 has
            std::vector<hipEvent_t> reached_u((size_t)n_units + 1, nullptr);
            struct Run { int64_t p0, s0, n; int64_t trig; };       // trig: in units
            std::deque<Run> pend;                         // movement tasks not yet issued, in list order
            std::vector<uint8_t> pending((size_t)N, 0);
            int64_t copy_at = 0;                          // logical time (units) the copy stream is known to have passed
            auto take = [&](int64_t want, std::vector<Run>* out) {
                while (want > 0 && !pend.empty()) {
                    Run& r = pend.front();
                    const int64_t n = r.n < want ? r.n : want;
                    out->push_back(Run{r.p0, r.s0, n, r.trig});
                    for (int64_t q = 0; q < n; ++q) pending[(size_t)(r.p0 + q)] = 0;
                    r.p0 += n;
                    r.s0 += n;
                    r.n -= n;
                    want -= n;
                    if (r.n == 0) pend.pop_front();
                }
            };
            // pages at the front of pend up to and including the last pending page of units [a, b]
            auto pages_through = [&](int64_t a, int64_t b) -> int64_t {
                if (b >= n_units) b = n_units - 1;
                if (a > b) return 0;
                int64_t last = -1;
                for (int64_t q = unit_first[(size_t)a]; q < unit_first[(size_t)b + 1]; ++q)
                    if (pending[(size_t)q]) last = q;
                if (last < 0) return 0;
                int64_t n = 0;
                for (const Run& r : pend) {
                    if (last >= r.p0 && last < r.p0 + r.n) return n + (last - r.p0 + 1);
                    n += r.n;
                }
                return n;
            };
            auto exchange = [&](const std::vector<Run>& in, const std::vector<Run>& out) -> int {
                int64_t trig = 0;
                for (const Run& r : in) trig = r.trig > trig ? r.trig : trig;
                if (trig > copy_at) {
                    APM_HIP(hipStreamWaitEvent(s_in, reached_u[(size_t)trig], 0));
                    copy_at = trig;
                }
                // pieces of equal page counts in the two directions, cut where either list's run ends,
                // so that every launch is busy both ways; what one list has left over goes alone
                size_t xi = 0, xo = 0;
                int64_t used_i = 0, used_o = 0;  // pages of the current runs already launched
                while (xi < in.size() || xo < out.size()) {
                    const int64_t left_i = xi < in.size() ? in[xi].n - used_i : 0;
                    const int64_t left_o = xo < out.size() ? out[xo].n - used_o : 0;
                    const int64_t n = left_i == 0 ? left_o : left_o == 0 ? left_i : (left_i < left_o ? left_i : left_o);
                    DuplexCopy d{};
                    d.used = dev->d_used;
                    d.page_bytes = (int64_t)pb;
                    d.host_store_policy = s->host_wt ? 3 : 0;
                    if (left_i > 0) {
                        const int64_t p0 = in[xi].p0 + used_i, s0 = in[xi].s0 + used_i;
                        for (int c = 0; c < 3; ++c) {
                            d.in_src[c] = reinterpret_cast<const char*>(s->host_dev[c]) + (size_t)p0 * pb;
                            d.in_dst[c] = reinterpret_cast<char*>(s->stage[c] + (size_t)s0 * (size_t)E);
                        }
                        d.in_bytes = (int64_t)(pb * (size_t)n);
                        d.in_first_page = p0;
                        used_i += n;
                        if (used_i == in[xi].n) { ++xi; used_i = 0; }
                    }
                    if (left_o > 0) {
                        const int64_t p0 = out[xo].p0 + used_o, s0 = out[xo].s0 + used_o;
                        for (int c = 0; c < 3; ++c) {
                            d.out_src[c] = reinterpret_cast<const char*>(s->stage[c] + (size_t)s0 * (size_t)E);
                            d.out_dst[c] = reinterpret_cast<char*>(s->host_dev[c]) + (size_t)p0 * pb;
                        }
                        d.out_bytes = (int64_t)(pb * (size_t)n);
                        d.out_first_page = p0;
                        used_o += n;
                        if (used_o == out[xo].n) { ++xo; used_o = 0; }
                    }
                    APM_HIP(launch_duplex_copy(d, s->direct_waves, s->direct_per_wg, s_in));
                }
                if (!in.empty()) {
                    hipEvent_t done;
                    int rc2 = new_event(&done);
                    if (rc2 != APM_OK) return rc2;
                    APM_HIP(hipEventRecord(done, s_in));
                    for (const Run& r : in)
                        for (int64_t q = 0; q < r.n; ++q) page_in[(size_t)(r.p0 + q)] = done;
                }
                return APM_OK;
            };
            int64_t k = 0;
            while (k < n_tasks) {
                if (tasks[k].op == APM_TASK_MOVE_TO_GPU) {
                    const int64_t p0 = tasks[k].target, s0 = slot_seq[(size_t)p0];
                    const int32_t trig = tasks[k].trigger_id;
                    int64_t n = 1;
                    while (k + n < n_tasks && tasks[k + n].op == APM_TASK_MOVE_TO_GPU && tasks[k + n].target == p0 + n &&
                           slot_seq[(size_t)(p0 + n)] == s0 + n && tasks[k + n].trigger_id == trig)
                        ++n;
                    pend.push_back(Run{p0, s0, n, first_unit[(size_t)trig]});
                    for (int64_t q = 0; q < n; ++q) pending[(size_t)(p0 + q)] = 1;
                    k += n;
                    continue;
                }
                const int64_t i = tasks[k].target;
                ++k;
                for (int64_t u = first_unit[(size_t)i]; u < first_unit[(size_t)i + 1]; ++u) {
                    {   // what this unit still waits for goes now, alone
                        std::vector<Run> in;
                        take(pages_through(u, u), &in);
                        rc = exchange(in, {});
                        if (rc != APM_OK) return rc;
                    }
                    hipEvent_t computed;
                    rc = compute_pages(unit_first[(size_t)u], unit_first[(size_t)u + 1] - unit_first[(size_t)u], &computed);
                    if (rc != APM_OK) return rc;
                    reached_u[(size_t)u + 1] = computed;
                    const std::vector<int64_t>& rel = unit_release[(size_t)u];
                    if (rel.empty()) continue;
                    std::vector<Run> out, in;
                    for (size_t j = 0; j < rel.size();) {  // runs of consecutive pages and slots
                        const int64_t q0 = rel[j], s0 = slot_seq[(size_t)q0];
                        size_t m = 1;
                        while (j + m < rel.size() && rel[j + m] == q0 + (int64_t)m && slot_seq[(size_t)rel[j + m]] == s0 + (int64_t)m) ++m;
                        out.push_back(Run{q0, s0, (int64_t)m, 0});
                        j += m;
                    }
                    // as many used elements in as go out (an exchange lasts as long as its longer
                    // direction), but at least what the next two units need
                    int64_t out_used = 0, in_used = 0, want = 0;
                    for (int64_t q : rel) out_used += dev->plan.pages[(size_t)q].used;
                    for (const Run& r : pend) {
                        for (int64_t q = 0; q < r.n && in_used < out_used; ++q, ++want)
                            in_used += dev->plan.pages[(size_t)(r.p0 + q)].used;
                        if (in_used >= out_used) break;
                    }
                    const int64_t ahead = pages_through(u + 1, u + 2);
                    take(ahead > want ? ahead : want, &in);
                    APM_HIP(hipStreamWaitEvent(s_in, computed, 0));
                    copy_at = u + 1;
                    rc = exchange(in, out);
                    if (rc != APM_OK) return rc;
                }
            }
            if (!pend.empty()) return fail(APM_ESTATE, "internal: movement tasks left over after the last compute");
        } else {
            int64_t copy_in_at = 0;  // the logical time the copy-in stream is known to have passed
            int64_t k = 0;
            while (k < n_tasks) {
                if (tasks[k].op == APM_TASK_MOVE_TO_GPU) {
                    // a run of movement tasks over consecutive pages and consecutive slots with one
                    // trigger id is one copy per class
                    const int64_t p0 = tasks[k].target, s0 = slot_seq[(size_t)p0];
                    const int32_t trig = tasks[k].trigger_id;
                    int64_t n = 1;
                    while (k + n < n_tasks && tasks[k + n].op == APM_TASK_MOVE_TO_GPU && tasks[k + n].target == p0 + n &&
                           slot_seq[(size_t)(p0 + n)] == s0 + n && tasks[k + n].trigger_id == trig)
                        ++n;
                    if (trig > copy_in_at) {  // the copy-in stream is in order: earlier waits still hold
                        APM_HIP(hipStreamWaitEvent(s_in, reached[(size_t)trig], 0));
                        copy_in_at = trig;
                    }
                    hipEvent_t last_wait = nullptr;
                    for (int64_t j = 0; j < n; ++j) {
                        hipEvent_t w = slot_free[(size_t)(s0 + j)];
                        if (w && w != last_wait) {
                            APM_HIP(hipStreamWaitEvent(s_in, w, 0));
                            last_wait = w;
                        }
                    }
                    for (int c = 0; c < 3; ++c) {
                        const char* src = static_cast<const char*>(host->base[states[c]]) + (size_t)p0 * pb;
                        APM_HIP(hipMemcpyAsync(s->stage[c] + (size_t)s0 * (size_t)E, src, pb * (size_t)n, hipMemcpyHostToDevice, s_in));
                    }
                    hipEvent_t done;
                    rc = new_event(&done);
                    if (rc != APM_OK) return rc;
                    APM_HIP(hipEventRecord(done, s_in));
                    for (int64_t j = 0; j < n; ++j) page_in[(size_t)(p0 + j)] = done;
                    k += n;
                    continue;
                }
                const int64_t i = tasks[k].target;
                ++k;
                hipEvent_t computed;
                rc = compute_layer(i, &computed);
                if (rc != APM_OK) return rc;
                const std::vector<int64_t>& rel = release_at[(size_t)i];
                if (rel.empty()) continue;
                hipEvent_t written;
                rc = new_event(&written);
                if (rc != APM_OK) return rc;
                APM_HIP(hipStreamWaitEvent(s_out, computed, 0));
                for (size_t j = 0; j < rel.size();) {  // write back in runs of consecutive pages and slots
                    const int64_t q0 = rel[j], s0 = slot_seq[(size_t)q0];
                    size_t m = 1;
                    while (j + m < rel.size() && rel[j + m] == q0 + (int64_t)m && slot_seq[(size_t)rel[j + m]] == s0 + (int64_t)m) ++m;
                    for (int c = 0; c < 3; ++c) {
                        char* dst = static_cast<char*>(host->base[states[c]]) + (size_t)q0 * pb;
                        APM_HIP(hipMemcpyAsync(dst, s->stage[c] + (size_t)s0 * (size_t)E, pb * m, hipMemcpyDeviceToHost, s_out));
                    }
                    j += m;
                }
                APM_HIP(hipEventRecord(written, s_out));
                for (int64_t q : rel) slot_free[(size_t)slot_seq[(size_t)q]] = written;
            }
        }
        rc = dev->ring.seal(slots_ring_slot, s->s_cmp);
        if (rc != APM_OK) return rc;
        // every copy-in feeds a compute and every page a write-back; the copy-out stream also waits
        // for the last compute, so it ends last
        if (last_computed) APM_HIP(hipStreamWaitEvent(s_out, last_computed, 0));
        APM_HIP(hipEventRecord(s->ev_done, s_out));
        APM_HIP(hipStreamWaitEvent(caller, s->ev_done, 0));
        return APM_OK;
    });
}

extern "C" int apm_streamer_copy_only(apm_streamer* s, int directions, void* stream) {
    return apm::guarded([&]() -> int {
        if (!s) return fail(APM_EINVAL, "NULL streamer");
        if (directions < 1 || directions > 3) return fail(APM_EINVAL, "directions must be 1 (H2D), 2 (D2H) or 3 (both)");
        return run_pipeline(s, directions, 1, nullptr, nullptr, nullptr, stream);
    });
}
