// Third tier: fp32 master / momentum / variance pages live in files (the Page listing's device
// map names SSD, Sec. 4.1; Alg. 2's updating actor fetches the states from SSD and offloads them
// back).  A small window of pinned host memory is the only staging: I/O threads read batch b+1..
// into free window slots and write finished batches back while the update kernel works on batch b
// directly in the window, across PCIe (the streamer's direct mode; no HBM staging, no copies).
//
// File I/O is not stream-ordered, so a step is driven from the host: the calling thread (or, for
// the one-step-stale form, the library's updater thread -- Alg. 2's two actors as two host
// threads) waits for a slot's reads, enqueues the kernels, waits for their event and hands the
// slot to the writers; the last write of a slot starts the reads of the batch that reuses it.
#include <cerrno>
#include <cstring>
#include <string>
#include <system_error>
#include <thread>

#include "apm_internal.h"
#include "apm_io.h"

using namespace apm;
using apm::io::IoPool;
using apm::io::WindowChain;
using apm::io::io_piece;

struct apm_tiered {
    apm_pool* file = nullptr;
    apm_pool* dev = nullptr;
    int64_t B = 0;
    int n_slots = 0;
    char* win[3] = {nullptr, nullptr, nullptr};      // pinned window, n_slots * B pages per class
    float* win_dev[3] = {nullptr, nullptr, nullptr};  // the same memory as the GPU addresses it
    hipStream_t s_cmp = nullptr;
    hipEvent_t ev_start = nullptr;
    std::vector<hipEvent_t> ev_done;  // per slot
    IoPool* io = nullptr;
    WindowChain* chain = nullptr;  // the batches' way through the window (apm_io.h)
    uint8_t* d_skip = nullptr;     // per page: skipped? (device; used when the caller passes no mask)
    uint8_t* h_skip = nullptr;     // the same on the host (pinned)
    int64_t first_page = 0;        // the step covers model pages [first_page, first_page + page_count)
    int64_t page_count = -1;       // -1 = to the last page in use
    StageRing ring;                // page lists of the batches; the handle's own, because the step may
                                   // run on the updater thread while the caller uses the GPU pool's

    // one-step-stale form
    std::thread updater;
    bool updater_running = false;
    int updater_rc = APM_OK;
    std::string updater_err;
    apm_hyper updater_hyper{};
};

namespace {

void free_tiered(apm_tiered* t) {
    if (t->updater.joinable()) t->updater.join();
    delete t->io;  // drains and joins the I/O threads
    delete t->chain;
    (void)hipDeviceSynchronize();
    for (char* p : t->win) if (p) (void)hipHostFree(p);
    t->ring.destroy();
    if (t->d_skip) (void)hipFree(t->d_skip);
    if (t->h_skip) (void)hipHostFree(t->h_skip);
    for (hipEvent_t e : t->ev_done) if (e) (void)hipEventDestroy(e);
    if (t->ev_start) (void)hipEventDestroy(t->ev_start);
    if (t->s_cmp) (void)hipStreamDestroy(t->s_cmp);
    delete t;
}

// One step; blocks until the last write has completed.  caller != nullptr: the kernels start after
// everything enqueued on that stream so far.
int tiered_run(apm_tiered* t, int64_t step, const apm_hyper* hyper, const uint16_t* g16_override,
               float* grad_norm, uint8_t* skip_mask, bool have_caller, hipStream_t caller) {
    apm_pool* dev = t->dev;
    AdamwLaunch L{};
    int rc = prepare_hyper(hyper, step, &L);
    if (rc != APM_OK) return rc;
    APM_HIP(hipSetDevice(dev->desc.hip_device));
    const int64_t in_use = (int64_t)dev->plan.pages.size();
    const int64_t P0 = t->first_page < in_use ? t->first_page : in_use;  // first model page of the step
    const int64_t N = t->page_count < 0 || t->page_count > in_use - P0 ? in_use - P0 : t->page_count;
    const int64_t E = dev->desc.page_elems;
    if (have_caller) {
        APM_HIP(hipEventRecord(t->ev_start, caller));
        APM_HIP(hipStreamWaitEvent(t->s_cmp, t->ev_start, 0));
    }
    L.g16 = g16_override ? g16_override : static_cast<const uint16_t*>(dev->base[APM_G16]);
    L.p16 = static_cast<uint16_t*>(dev->base[APM_P16]);
    L.used = dev->d_used;
    L.E = E;
    L.S = dev->S;
    L.p32 = t->win_dev[0];
    L.m32 = t->win_dev[1];
    L.v32 = t->win_dev[2];
    L.meta = dev->d_meta;
    L.stride_wavefronts = kDirectWavefronts;
    L.stride_waves_per_wg = 1;
    const bool need_reduce = grad_norm || skip_mask || L.max_norm > 0.0 || L.skip_mode != APM_SKIP_NONE;
    if (need_reduce) {
        L.partials = dev->d_partials;
        L.nzflags = dev->d_nzflags;
    }
    // With skipping on, a page without gradient needs no I/O at all: one reduce pass over every page
    // (the gradients are in HBM: 2 B per element) decides which pages are skipped -- and writes the
    // caller's per-page outputs -- and only the other pages pass through the window.
    std::vector<int64_t> active;
    const bool sparse = L.skip_mode == APM_SKIP_UNTOUCHED && N > 0;
    if (sparse) {
        AdamwLaunch A = L;
        A.state_first = A.grad_first = P0;
        A.n_listed = N;
        A.grad_norm = grad_norm ? grad_norm + P0 : nullptr;
        A.skip_mask = skip_mask ? skip_mask + P0 : t->d_skip;
        APM_HIP(launch_grad_reduce(A, t->s_cmp));
        APM_HIP(hipMemcpyAsync(t->h_skip, A.skip_mask, (size_t)N, hipMemcpyDefault, t->s_cmp));
        APM_HIP(hipStreamSynchronize(t->s_cmp));
        for (int64_t p = 0; p < N; ++p)
            if (!t->h_skip[p]) active.push_back(P0 + p);
    } else if (P0 > 0) {  // a range that does not start at page 0 goes through the list form as well
        active.resize((size_t)N);
        for (int64_t p = 0; p < N; ++p) active[(size_t)p] = P0 + p;
    }
    const bool listed = sparse || P0 > 0;
    // Kernels are skipped after a failure, but every batch still passes through the chain so that
    // the step drains.
    hipError_t gpu_err = hipSuccess;
    int ring_rc = APM_OK;
    const auto process = [&](int64_t, int slot, int64_t first, int64_t nb) {
        AdamwLaunch C = L;
        C.state_first = (int64_t)slot * t->B;
        C.n_listed = nb;
        int ring_slot = -1;
        if (sparse) {  // list positions [first, first + nb) of the active pages; outputs are written already
            ring_rc = t->ring.acquire((size_t)nb * sizeof(int64_t), &ring_slot);
            if (ring_rc != APM_OK) return false;
            int64_t* h = static_cast<int64_t*>(t->ring.h[ring_slot]);
            for (int64_t k = 0; k < nb; ++k) h[k] = active[(size_t)(first + k)];
            ring_rc = t->ring.commit(ring_slot, (size_t)nb * sizeof(int64_t), t->s_cmp);
            if (ring_rc != APM_OK) return false;
            C.grad_pages = static_cast<const int64_t*>(t->ring.d[ring_slot]);
        } else {  // consecutive model pages from P0 + first on
            C.grad_first = P0 + first;
            C.grad_norm = grad_norm ? grad_norm + P0 + first : nullptr;
            C.skip_mask = skip_mask ? skip_mask + P0 + first : nullptr;
        }
        gpu_err = need_reduce ? launch_grad_reduce(C, t->s_cmp) : launch_prepare(C, t->s_cmp);
        if (gpu_err == hipSuccess) gpu_err = launch_adamw(C, t->s_cmp);
        if (gpu_err == hipSuccess) gpu_err = hipEventRecord(t->ev_done[(size_t)slot], t->s_cmp);
        if (gpu_err == hipSuccess) gpu_err = hipEventSynchronize(t->ev_done[(size_t)slot]);
        if (ring_slot >= 0 && gpu_err == hipSuccess) ring_rc = t->ring.seal(ring_slot, t->s_cmp);
        return gpu_err == hipSuccess && ring_rc == APM_OK;
    };
    const int io_err = listed ? t->chain->run_list(active.data(), (int64_t)active.size(), process)
                              : t->chain->run(N, process);
    if (io_err > 0) return fail(APM_EDEVICE, "file I/O failed during the step: %s (the files may hold a partly updated state)", strerror(io_err));
    if (gpu_err != hipSuccess) return fail(APM_EDEVICE, "a kernel launch of the step failed: %s", hipGetErrorString(gpu_err));
    return ring_rc;
}

int join_updater(apm_tiered* t) {
    if (!t->updater_running) return APM_OK;
    t->updater.join();
    t->updater_running = false;
    if (t->updater_rc != APM_OK) return fail(t->updater_rc, "the background update failed: %s", t->updater_err.c_str());
    return APM_OK;
}

}  // namespace

extern "C" int apm_file_pool_create(apm_pool** out, const char* path_prefix, int32_t hip_device,
                                    int64_t page_elems, int64_t n_pages, uint32_t state_mask,
                                    uint32_t flags) {
    return apm::guarded([&]() -> int {
        if (!out || !path_prefix || !*path_prefix) return fail(APM_EINVAL, "NULL argument or empty path prefix");
        if (page_elems <= 0 || page_elems % kAlign != 0 || page_elems > (int64_t)1 << 30) return fail(APM_EINVAL, "page_elems must be a positive multiple of %lld, at most 2^30", (long long)kAlign);
        if (n_pages <= 0) return fail(APM_EINVAL, "n_pages must be positive");
        if (state_mask == 0 || state_mask >> APM_N_STATES) return fail(APM_EINVAL, "bad state_mask 0x%x", state_mask);
        if (flags & ~(uint32_t)(APM_POOL_NO_ZERO | APM_POOL_FILE_DIRECT)) return fail(APM_EINVAL, "unknown flags 0x%x", flags);
        apm_pool* pool = new apm_pool();
        pool->desc.device = APM_DEV_FILE;
        pool->desc.hip_device = hip_device;
        pool->desc.page_elems = page_elems;
        pool->desc.n_pages = n_pages;
        pool->desc.state_mask = state_mask;
        pool->desc.flags = flags;
        static const char* const suffix[APM_N_STATES] = {".p32", ".m32", ".v32", ".g16", ".p16"};
        for (int st = 0; st < APM_N_STATES; ++st) {
            if (!pool->stores(st)) continue;
            const size_t page_bytes = (size_t)page_elems * (size_t)elem_bytes(st);
            if ((flags & APM_POOL_FILE_DIRECT) && page_bytes % 4096 != 0) {
                apm_pool_destroy(pool);
                return fail(APM_EINVAL, "unbuffered file I/O needs pages of a multiple of 4096 bytes (class %d has %zu)", st, page_bytes);
            }
            const std::string path = std::string(path_prefix) + suffix[st];
            int oflags = O_RDWR | O_CREAT | O_CLOEXEC;
            if (!(flags & APM_POOL_NO_ZERO)) oflags |= O_TRUNC;  // recreated at full size below: reads as zeros
            if (flags & APM_POOL_FILE_DIRECT) oflags |= O_DIRECT;
            const int fd = open(path.c_str(), oflags, 0600);
            if (fd < 0 || ftruncate(fd, (off_t)(page_bytes * (size_t)n_pages)) != 0) {
                const int err = errno;
                if (fd >= 0) close(fd);
                apm_pool_destroy(pool);
                return fail(APM_EDEVICE, "cannot create %s: %s", path.c_str(), strerror(err));
            }
            pool->fd[st] = fd;
        }
        *out = pool;
        return APM_OK;
    });
}

namespace apm {
// FILE <-> HOST page copy, done before returning (file I/O is not stream-ordered; the caller's
// stream is synchronised first so that the host pages are what the stream left there).
int file_page_copy(apm_pool* dst, int64_t dst_page, apm_pool* src, int64_t src_page, int64_t n_pages,
                   int state, hipStream_t stream) {
    apm_pool* file = dst->desc.device == APM_DEV_FILE ? dst : src;
    apm_pool* host = dst->desc.device == APM_DEV_FILE ? src : dst;
    if (host->desc.device != APM_DEV_HOST) return fail(APM_EDEVICE, "a FILE pool exchanges pages with HOST pools only");
    const bool write = file == dst;
    APM_HIP(hipSetDevice(host->desc.hip_device));
    APM_HIP(hipStreamSynchronize(stream));
    const size_t pb = (size_t)file->desc.page_elems * (size_t)elem_bytes(state);
    char* buf = static_cast<char*>(host->base[state]) + (size_t)(write ? src_page : dst_page) * pb;
    const off_t off = (off_t)((size_t)(write ? dst_page : src_page) * pb);
    const int err = io_piece(file->fd[state], buf, pb * (size_t)n_pages, off, write,
                             (file->desc.flags & APM_POOL_FILE_DIRECT) != 0);
    if (err) return fail(APM_EDEVICE, "file %s of %lld pages failed: %s", write ? "write" : "read", (long long)n_pages, strerror(err));
    return APM_OK;
}
}  // namespace apm

extern "C" int apm_tiered_create(apm_tiered** out, apm_pool* file, apm_pool* dev, int64_t batch_pages,
                                 int n_slots, int io_threads) {
    return apm::guarded([&]() -> int {
        if (!out || !file || !dev) return fail(APM_EINVAL, "NULL argument");
        if (file->desc.device != APM_DEV_FILE || dev->desc.device != APM_DEV_GPU) return fail(APM_EDEVICE, "expected a FILE pool and a GPU pool");
        for (int st : {APM_P32, APM_M32, APM_V32}) if (!file->stores(st)) return fail(APM_ESTATE, "file pool lacks fp32 class %d", st);
        for (int st : {APM_G16, APM_P16}) if (!dev->stores(st)) return fail(APM_ESTATE, "GPU pool lacks 16-bit class %d", st);
        if (file->desc.page_elems != dev->desc.page_elems) return fail(APM_EINVAL, "pools have different page sizes");
        if (file->desc.n_pages < dev->desc.n_pages) return fail(APM_EINVAL, "file pool has fewer pages than the GPU pool");
        if (batch_pages < 1 || batch_pages > dev->desc.n_pages) return fail(APM_EINVAL, "batch_pages out of range");
        if (n_slots < 2 || n_slots > 64) return fail(APM_EINVAL, "n_slots must be in [2, 64]");
        if (io_threads < 1 || io_threads > 64) return fail(APM_EINVAL, "io_threads must be in [1, 64]");
        APM_HIP(hipSetDevice(dev->desc.hip_device));
        apm_tiered* t = new apm_tiered();
        t->file = file; t->dev = dev; t->B = batch_pages; t->n_slots = n_slots;
        const size_t bytes = (size_t)n_slots * (size_t)batch_pages * (size_t)dev->desc.page_elems * sizeof(float);
        hipError_t e = hipSuccess;
        for (int k = 0; k < 3 && e == hipSuccess; ++k) {
            e = hipHostMalloc((void**)&t->win[k], bytes, hipHostMallocDefault);
            if (e == hipSuccess) e = hipHostGetDevicePointer((void**)&t->win_dev[k], t->win[k], 0);
        }
        if (e != hipSuccess) {
            (void)hipGetLastError();
            free_tiered(t);
            return fail(APM_ENOMEM, "allocating 3 x %zu bytes of pinned window failed: %s", bytes, hipGetErrorString(e));
        }
        e = hipStreamCreateWithFlags(&t->s_cmp, hipStreamNonBlocking);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&t->ev_start, hipEventDisableTiming);
        t->ev_done.assign((size_t)n_slots, nullptr);
        for (int k = 0; k < n_slots && e == hipSuccess; ++k) e = hipEventCreateWithFlags(&t->ev_done[(size_t)k], hipEventDisableTiming);
        if (e != hipSuccess) {
            free_tiered(t);
            return fail(APM_EDEVICE, "creating the stream / events failed: %s", hipGetErrorString(e));
        }
        e = hipMalloc((void**)&t->d_skip, (size_t)dev->desc.n_pages);
        if (e == hipSuccess) e = hipHostMalloc((void**)&t->h_skip, (size_t)dev->desc.n_pages, hipHostMallocDefault);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            free_tiered(t);
            return fail(APM_ENOMEM, "allocating the per-page skip flags failed: %s", hipGetErrorString(e));
        }
        int rc = ensure_scratch(dev);
        if (rc != APM_OK) { free_tiered(t); return rc; }
        try {
            t->io = new IoPool(io_threads);
            const int fds[3] = {file->fd[APM_P32], file->fd[APM_M32], file->fd[APM_V32]};
            t->chain = new WindowChain(t->io, fds, t->win, (size_t)dev->desc.page_elems * sizeof(float), batch_pages,
                                       n_slots, (file->desc.flags & APM_POOL_FILE_DIRECT) != 0);
        } catch (...) {  // threads or memory ran out: give back what the handle holds, report through the guard
            free_tiered(t);
            throw;
        }
        *out = t;
        return APM_OK;
    });
}

extern "C" int apm_tiered_destroy(apm_tiered* t) {
    return apm::guarded([&]() -> int {
        if (!t) return APM_OK;
        (void)hipSetDevice(t->dev->desc.hip_device);
        free_tiered(t);
        return APM_OK;
    });
}

extern "C" int apm_tiered_set_range(apm_tiered* t, int64_t first_page, int64_t n_pages) {
    return apm::guarded([&]() -> int {
        if (!t) return fail(APM_EINVAL, "NULL handle");
        if (first_page < 0 || first_page > t->dev->desc.n_pages) return fail(APM_ERANGE, "first_page out of range");
        int rc = join_updater(t);
        if (rc != APM_OK) return rc;
        t->first_page = first_page;
        t->page_count = n_pages < 0 ? -1 : n_pages;
        return APM_OK;
    });
}

extern "C" int apm_tiered_io_bytes(apm_tiered* t, int64_t* bytes_read, int64_t* bytes_written) {
    return apm::guarded([&]() -> int {
        if (!t) return fail(APM_EINVAL, "NULL handle");
        t->chain->io_bytes(bytes_read, bytes_written);
        return APM_OK;
    });
}

extern "C" int apm_tiered_step(apm_tiered* t, int64_t step, const apm_hyper* hyper, float* grad_norm,
                               uint8_t* skip_mask, void* stream) {
    return apm::guarded([&]() -> int {
        if (!t) return fail(APM_EINVAL, "NULL handle");
        if (!t->dev->has_layout) return fail(APM_ESTATE, "the GPU pool has no layout");
        int rc = join_updater(t);
        if (rc != APM_OK) return rc;
        return tiered_run(t, step, hyper, nullptr, grad_norm, skip_mask, true, static_cast<hipStream_t>(stream));
    });
}

extern "C" int apm_tiered_step_delayed(apm_tiered* t, const void* new_g16, const apm_hyper* hyper,
                                       void* stream) {
    return apm::guarded([&]() -> int {
        if (!t) return fail(APM_EINVAL, "NULL handle");
        apm_pool* dev = t->dev;
        if (!dev->has_layout) return fail(APM_ESTATE, "the GPU pool has no layout");
        AdamwLaunch probe{};
        int rc = prepare_hyper(hyper, 1, &probe);  // validate before any state changes
        if (rc != APM_OK) return rc;
        APM_HIP(hipSetDevice(dev->desc.hip_device));
        rc = ensure_delayed(dev, nullptr, false);  // the updater is a host thread here: no stream to pair
        if (rc != APM_OK) return rc;
        for (int k = 0; k < 2 && new_g16; ++k)  // the updater reads the halves with no stream-side guard
            if (new_g16 == static_cast<const void*>(dev->gbuf[k])) return fail(APM_EINVAL, "the zero-copy hand-over (apm_delayed_grad_buffer) is not available with file-resident state: pass the producer's own buffer");
        // One updater at a time: the update handed over by the previous call must have finished
        // before the next one starts (and before the half it read is staged into again).
        rc = join_updater(t);
        if (rc != APM_OK) return rc;
        hipStream_t s = static_cast<hipStream_t>(stream);
        if (dev->buffered) {
            const int k = dev->cur;
            t->updater_hyper = dev->buf_hyper;  // the values the buffered gradient was handed over with
            const int64_t step_no = dev->applied + 1;
            const uint16_t* g16 = dev->gbuf[k];
            hipEvent_t staged = dev->ev_staged[k];
            float* norm = dev->delayed_norm;
            uint8_t* skip = dev->delayed_skip;
            try {
                t->updater = std::thread([t, step_no, g16, staged, norm, skip] {
                    // Alg. 2's updating actor: waits for the handed-over gradient, then fetches, updates
                    // and offloads the states batch by batch.
                    t->updater_rc = guarded([&]() -> int {
                        if (hipSetDevice(t->dev->desc.hip_device) != hipSuccess || hipEventSynchronize(staged) != hipSuccess)
                            return fail(APM_EDEVICE, "waiting for the staged gradient failed");
                        return tiered_run(t, step_no, &t->updater_hyper, g16, norm, skip, false, nullptr);
                    });
                    if (t->updater_rc != APM_OK) t->updater_err = apm_last_error();
                });
            } catch (const std::system_error& e) {  // nothing has changed: the gradient stays buffered
                return fail(APM_EDEVICE, "starting the updater thread failed: %s", e.what());
            }
            t->updater_running = true;
            dev->applied = step_no;
            dev->buffered = false;
        }
        if (!new_g16) return join_updater(t);  // flush: the update has completed when this returns
        const int nxt = dev->cur ^ 1;
        const int64_t N = (int64_t)dev->plan.pages.size();
        const size_t bytes = (size_t)N * (size_t)dev->desc.page_elems * 2u;
        APM_HIP(hipMemcpyAsync(dev->gbuf[nxt], new_g16, bytes, hipMemcpyDeviceToDevice, s));
        APM_HIP(hipEventRecord(dev->ev_staged[nxt], s));
        dev->buf_hyper = *hyper;
        dev->buf_pages.clear();
        dev->buf_pages_null = true;
        dev->buf_n_pages = N;
        dev->cur = nxt;
        dev->buffered = true;
        return APM_OK;
    });
}
