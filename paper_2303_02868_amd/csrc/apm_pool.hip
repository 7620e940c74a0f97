// Page pool, page table, pack / unpack entry points and page copies (host side).
#include <cstring>
#include <thread>

#include <unistd.h>

#include "apm_internal.h"

namespace apm {

// ---- staging ring -------------------------------------------------------------------------
int StageRing::acquire(size_t bytes, int* slot) {
    const int k = next;
    next = (next + 1) % K;
    if (busy[k]) {
        APM_HIP(hipEventSynchronize(ev[k]));
        busy[k] = false;
    }
    if (cap[k] < bytes) {
        if (h[k]) APM_HIP(hipHostFree(h[k]));
        if (d[k]) APM_HIP(hipFree(d[k]));
        h[k] = d[k] = nullptr;
        cap[k] = 0;
        size_t want = 65536;
        while (want < bytes) want *= 2;
        APM_HIP(hipHostMalloc(&h[k], want, hipHostMallocDefault));
        APM_HIP(hipMalloc(&d[k], want));
        cap[k] = want;
    }
    if (!ev[k]) APM_HIP(hipEventCreateWithFlags(&ev[k], hipEventDisableTiming));
    *slot = k;
    return APM_OK;
}

int StageRing::commit(int k, size_t bytes, hipStream_t s) {
    APM_HIP(hipMemcpyAsync(d[k], h[k], bytes, hipMemcpyHostToDevice, s));
    APM_HIP(hipEventRecord(ev[k], s));
    busy[k] = true;
    return APM_OK;
}

int StageRing::seal(int k, hipStream_t s) {
    APM_HIP(hipEventRecord(ev[k], s));
    busy[k] = true;
    return APM_OK;
}

void StageRing::destroy() {
    for (int k = 0; k < K; ++k) {
        if (busy[k]) (void)hipEventSynchronize(ev[k]);
        if (ev[k]) (void)hipEventDestroy(ev[k]);
        if (h[k]) (void)hipHostFree(h[k]);
        if (d[k]) (void)hipFree(d[k]);
        h[k] = d[k] = nullptr;
        ev[k] = nullptr;
        cap[k] = 0;
        busy[k] = false;
    }
}

int ensure_scratch(apm_pool* pool) {
    if (pool->d_partials && pool->d_nzflags && pool->d_meta) return APM_OK;
    const size_t n = (size_t)pool->desc.n_pages * (size_t)pool->S;
    auto get = [](void** p, size_t bytes) -> int {  // a buffer an earlier, failed attempt got is kept
        if (*p) return APM_OK;
        hipError_t e = hipMalloc(p, bytes);
        if (e == hipSuccess) return APM_OK;
        (void)hipGetLastError();
        *p = nullptr;
        return fail(APM_ENOMEM, "allocating %zu bytes of per-page scratch failed: %s", bytes, hipGetErrorString(e));
    };
    int rc = get((void**)&pool->d_partials, n * sizeof(double));
    if (rc == APM_OK) rc = get((void**)&pool->d_nzflags, n * sizeof(uint32_t));
    if (rc == APM_OK) rc = get((void**)&pool->d_meta, (size_t)pool->desc.n_pages * sizeof(PageMeta));
    return rc;
}

namespace {

size_t region_bytes(const apm_pool* p, int state) {
    return (size_t)p->desc.n_pages * (size_t)p->desc.page_elems * (size_t)elem_bytes(state);
}

int zero_regions(apm_pool* pool, hipStream_t s, bool at_create) {
    for (int st = 0; st < APM_N_STATES; ++st) {
        if (!pool->stores(st)) continue;
        if (at_create && (pool->desc.flags & APM_POOL_NO_ZERO)) continue;
        if (pool->desc.device == APM_DEV_HOST) {
            APM_HIP(hipStreamSynchronize(s));
            // a host region can be ~100 GB: spread the page-touching over a few threads
            const size_t bytes = region_bytes(pool, st);
            const size_t n_thr = bytes >= ((size_t)1 << 30) ? 8 : 1;
            const size_t per = (bytes / n_thr + 4095) / 4096 * 4096;
            std::vector<std::thread> thr;
            char* base = static_cast<char*>(pool->base[st]);
            for (size_t k = 0; k < n_thr; ++k) {
                const size_t a = k * per < bytes ? k * per : bytes;
                const size_t b = (k + 1) * per < bytes ? (k + 1) * per : bytes;
                if (b > a) thr.emplace_back([=] { std::memset(base + a, 0, b - a); });
            }
            for (auto& t : thr) t.join();
        } else {
            APM_HIP(hipMemsetAsync(pool->base[st], 0, region_bytes(pool, st), s));
        }
    }
    return APM_OK;
}

void free_pool(apm_pool* pool) {
    for (int st = 0; st < APM_N_STATES; ++st)
        if (pool->fd[st] >= 0) (void)close(pool->fd[st]);
    for (int st = 0; st < APM_N_STATES; ++st) {
        if (pool->owned[st] && pool->alloc[st]) {
            if (pool->desc.device == APM_DEV_HOST) (void)hipHostFree(pool->alloc[st]);
            else (void)hipFree(pool->alloc[st]);
        }
    }
    if (pool->d_used) (void)hipFree(pool->d_used);
    if (pool->d_partials) (void)hipFree(pool->d_partials);
    if (pool->d_nzflags) (void)hipFree(pool->d_nzflags);
    if (pool->d_meta) (void)hipFree(pool->d_meta);
    pool->ring.destroy();
    for (auto& t : pool->timed) {
        (void)hipEventDestroy(t.begin);
        (void)hipEventDestroy(t.end);
    }
    for (int k = 0; k < 2; ++k) {
        if (pool->gbuf[k]) (void)hipFree(pool->gbuf[k]);
        if (pool->ev_staged[k]) (void)hipEventDestroy(pool->ev_staged[k]);
        if (pool->ev_applied[k]) (void)hipEventDestroy(pool->ev_applied[k]);
    }
    if (pool->ev_flush) (void)hipEventDestroy(pool->ev_flush);
    if (pool->upd_stream) (void)hipStreamDestroy(pool->upd_stream);
    delete pool;
}

int install_layout(apm_pool* pool, const apm_tensor* tensors, int64_t n, Plan&& plan, hipStream_t s) {
    if ((int64_t)plan.pages.size() > pool->desc.n_pages)
        return fail(APM_ENOMEM, "layout needs %lld pages, pool has %lld", (long long)plan.pages.size(), (long long)pool->desc.n_pages);
    if (pool->has_layout) {  // a different layout replaces the old one: old contents would alias
        int rc = zero_regions(pool, s, false);
        if (rc != APM_OK) return rc;
    }
    std::vector<int32_t> used((size_t)pool->desc.n_pages, 0);
    for (size_t k = 0; k < plan.pages.size(); ++k) used[k] = (int32_t)plan.pages[k].used;
    // The page table changes rarely; a synchronous upload keeps its lifetime trivial.
    APM_HIP(hipStreamSynchronize(s));
    APM_HIP(hipMemcpy(pool->d_used, used.data(), used.size() * sizeof(int32_t), hipMemcpyHostToDevice));
    pool->layout_numels.resize((size_t)n);
    pool->layout_ids.resize((size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        pool->layout_numels[(size_t)i] = tensors[i].numel;
        pool->layout_ids[(size_t)i] = tensors[i].id;
    }
    pool->plan = std::move(plan);
    pool->has_layout = true;
    return APM_OK;
}

bool same_layout(const apm_pool* pool, const apm_tensor* tensors, int64_t n) {
    if (!pool->has_layout || (int64_t)pool->layout_numels.size() != n) return false;
    for (int64_t i = 0; i < n; ++i)
        if (pool->layout_numels[(size_t)i] != tensors[i].numel) return false;
    return true;
}

int check_list(const apm_tensor* tensors, int64_t n) {
    if (n < 0 || (n > 0 && !tensors)) return fail(APM_EINVAL, "bad tensor list");
    return APM_OK;
}

int plan_of(const apm_pool* pool, const apm_tensor* tensors, int64_t n, Plan* out) {
    std::vector<int64_t> numels((size_t)n);
    for (int64_t i = 0; i < n; ++i) numels[(size_t)i] = tensors[i].numel;
    return make_plan(pool->desc.page_elems, numels.data(), n, out);
}

// Shared body of pack (to_pages) and unpack: one descriptor per segment, one kernel.
int move_segments(apm_pool* pool, int state, const apm_tensor* tensors, int64_t n, bool to_pages,
                  hipStream_t s) {
    const int eb = elem_bytes(state);
    const int want = state <= APM_V32 ? APM_F32 : APM_BF16;
    for (int64_t i = 0; i < n; ++i) {
        if (tensors[i].numel == 0) continue;
        if (tensors[i].dtype != want) return fail(APM_EINVAL, "tensor %lld: dtype %d does not match state class %d", (long long)i, tensors[i].dtype, state);
        if (!tensors[i].data) return fail(APM_EINVAL, "tensor %lld has no data pointer", (long long)i);
    }
    const auto& segs = pool->plan.segs;
    if (segs.empty()) return APM_OK;
    int slot;
    int rc = pool->ring.acquire(segs.size() * sizeof(SegDesc), &slot);
    if (rc != APM_OK) return rc;
    SegDesc* h = static_cast<SegDesc*>(pool->ring.h[slot]);
    char* region = static_cast<char*>(pool->base[state]);
    int64_t max_bytes = 0;
    for (size_t k = 0; k < segs.size(); ++k) {
        const apm_segment& g = segs[k];
        char* in_tensor = static_cast<char*>(tensors[g.tensor].data) + g.tensor_off * eb;
        char* in_page = region + (g.page * pool->desc.page_elems + g.page_off) * eb;
        h[k].src = to_pages ? in_tensor : in_page;
        h[k].dst = to_pages ? in_page : in_tensor;
        h[k].nbytes = g.n * eb;
        if (h[k].nbytes > max_bytes) max_bytes = h[k].nbytes;
    }
    rc = pool->ring.commit(slot, segs.size() * sizeof(SegDesc), s);
    if (rc != APM_OK) return rc;
    {
        ScopedTiming t(pool, APM_K_SEGCOPY, s);
        APM_HIP(launch_seg_copy(static_cast<const SegDesc*>(pool->ring.d[slot]), (int64_t)segs.size(), max_bytes, s));
    }
    return pool->ring.seal(slot, s);
}

}  // namespace
}  // namespace apm

using namespace apm;

extern "C" int apm_pool_create(apm_pool** out, const apm_pool_desc* desc) {
    return apm::guarded([&]() -> int {
        if (!out || !desc) return fail(APM_EINVAL, "NULL argument");
        if (desc->device != APM_DEV_GPU && desc->device != APM_DEV_HOST) return fail(APM_EINVAL, "unknown device kind %d", desc->device);
        if (desc->page_elems <= 0 || desc->page_elems % kAlign != 0) return fail(APM_EINVAL, "page_elems must be a positive multiple of %lld", (long long)kAlign);
        if (desc->page_elems > (int64_t)1 << 30) return fail(APM_EINVAL, "page_elems above 2^30 is not supported");
        if (desc->n_pages <= 0) return fail(APM_EINVAL, "n_pages must be positive");
        if (desc->n_pages > INT32_MAX || desc->n_pages > ((int64_t)1 << 60) / desc->page_elems) return fail(APM_EINVAL, "n_pages = %lld is beyond what a pool can index", (long long)desc->n_pages);
        if (desc->state_mask == 0 || desc->state_mask >> APM_N_STATES) return fail(APM_EINVAL, "bad state_mask 0x%x", desc->state_mask);
        for (int st = 0; st < APM_N_STATES; ++st)
            if (desc->base[st] && (reinterpret_cast<uintptr_t>(desc->base[st]) & 15u)) return fail(APM_EINVAL, "base[%d] is not 16-byte aligned", st);
        int n_dev = 0;
        APM_HIP(hipGetDeviceCount(&n_dev));
        if (desc->hip_device < 0 || desc->hip_device >= n_dev) return fail(APM_EDEVICE, "HIP device %d not present (%d visible)", desc->hip_device, n_dev);
        APM_HIP(hipSetDevice(desc->hip_device));

        apm_pool* pool = new apm_pool();
        pool->desc = *desc;
        pool->S = (int32_t)((desc->page_elems + kReduceTile - 1) / kReduceTile);
        for (int st = 0; st < APM_N_STATES; ++st) {
            if (!pool->stores(st)) { pool->desc.base[st] = nullptr; continue; }
            if (desc->base[st]) { pool->base[st] = desc->base[st]; continue; }
            // The class regions of a GPU pool start at different offsets modulo 8 KiB.  Element i of
            // every class is touched by the same wavefront at the same time; with identically aligned
            // regions its 4 KiB fp32 tiles all fall on the same memory channel.  Measured on MI355X
            // (update kernel, 1024 full pages): equal alignment or skews that are even multiples of
            // 4 KiB 5.95-6.0 TB/s, odd multiples 6.2-6.3 TB/s, the offsets below 6.31 TB/s.
            static const size_t kSkew[APM_N_STATES] = {0, 4096, 12288, 24576, 40960};
            const size_t skew = desc->device == APM_DEV_GPU ? kSkew[st] : 0;
            void* p = nullptr;
            hipError_t e = desc->device == APM_DEV_HOST ? hipHostMalloc(&p, region_bytes(pool, st), hipHostMallocDefault)
                                                        : hipMalloc(&p, region_bytes(pool, st) + skew);
            if (e != hipSuccess) {
                (void)hipGetLastError();
                const size_t wanted = region_bytes(pool, st);
                free_pool(pool);
                return fail(APM_ENOMEM, "allocating %zu bytes of %s memory for state class %d failed: %s", wanted,
                            desc->device == APM_DEV_HOST ? "pinned host" : "device", st, hipGetErrorString(e));
            }
            pool->alloc[st] = p;
            pool->base[st] = static_cast<char*>(p) + skew;
            pool->owned[st] = true;
        }
        hipError_t e = hipMalloc((void**)&pool->d_used, (size_t)desc->n_pages * sizeof(int32_t));
        if (e == hipSuccess) e = hipMemset(pool->d_used, 0, (size_t)desc->n_pages * sizeof(int32_t));
        if (e != hipSuccess) {
            free_pool(pool);
            return fail(APM_ENOMEM, "page table allocation failed: %s", hipGetErrorString(e));
        }
        int rc = zero_regions(pool, nullptr, true);
        if (rc == APM_OK && hipStreamSynchronize(nullptr) != hipSuccess) rc = fail(APM_EDEVICE, "zero-fill failed");
        if (rc != APM_OK) {
            free_pool(pool);
            return rc;
        }
        *out = pool;
        return APM_OK;
    });
}

extern "C" int apm_pool_destroy(apm_pool* pool) {
    return apm::guarded([&]() -> int {
        if (!pool) return APM_OK;
        if (pool->desc.device == APM_DEV_FILE) {  // holds file descriptors only: no HIP call
            free_pool(pool);
            return APM_OK;
        }
        (void)hipSetDevice(pool->desc.hip_device);
        if (pool->upd_stream) (void)hipStreamSynchronize(pool->upd_stream);
        hipError_t e = hipDeviceSynchronize();
        free_pool(pool);
        if (e != hipSuccess) return fail(APM_EDEVICE, "device synchronize failed: %s", hipGetErrorString(e));
        return APM_OK;
    });
}

extern "C" int64_t apm_pool_pages_in_use(const apm_pool* pool) {
    return pool && pool->has_layout ? (int64_t)pool->plan.pages.size() : 0;
}

extern "C" int apm_pool_page_info(const apm_pool* pool, int64_t page, apm_page_info* out) {
    return apm::guarded([&]() -> int {
        if (!pool || !out) return fail(APM_EINVAL, "NULL argument");
        if (page < 0 || page >= pool->desc.n_pages) return fail(APM_ERANGE, "page %lld out of range [0, %lld)", (long long)page, (long long)pool->desc.n_pages);
        apm_page_info info{};
        info.total_elems = pool->desc.page_elems;
        info.device = pool->desc.device;
        info.tensor_id[0] = info.tensor_id[1] = -1;
        if (pool->has_layout && page < (int64_t)pool->plan.pages.size()) {
            const PageEntry& e = pool->plan.pages[(size_t)page];
            info.used_elems = e.used;
            info.n_tensors = e.n_tensors;
            for (int k = 0; k < e.n_tensors; ++k) {
                info.tensor_id[k] = pool->layout_ids[(size_t)e.tensor[k]];
                info.tensor_elems[k] = e.tensor_elems[k];
            }
        }
        info.available_elems = info.total_elems - info.used_elems;
        *out = info;
        return APM_OK;
    });
}

extern "C" void* apm_pool_state_ptr(const apm_pool* pool, int state, int64_t page) {
    if (!pool || !pool->stores(state) || page < 0 || page >= pool->desc.n_pages) return nullptr;
    if (pool->desc.device == APM_DEV_FILE) return nullptr;
    return static_cast<char*>(pool->base[state]) + page * pool->desc.page_elems * elem_bytes(state);
}

extern "C" int apm_pool_set_layout(apm_pool* pool, const apm_tensor* tensors, int64_t n,
                                   apm_segment* segs, int64_t* n_segs, int64_t* n_pages,
                                   double* fragmentation, void* stream) {
    return apm::guarded([&]() -> int {
        if (!pool) return fail(APM_EINVAL, "NULL pool");
        if (pool->desc.device == APM_DEV_FILE) return fail(APM_EDEVICE, "a FILE pool takes its layout from the GPU pool it is used with");
        int rc = check_list(tensors, n);
        if (rc != APM_OK) return rc;
        APM_HIP(hipSetDevice(pool->desc.hip_device));
        if (!same_layout(pool, tensors, n)) {
            Plan plan;
            rc = plan_of(pool, tensors, n, &plan);
            if (rc != APM_OK) return rc;
            rc = install_layout(pool, tensors, n, std::move(plan), static_cast<hipStream_t>(stream));
            if (rc != APM_OK) return rc;
        } else {
            for (int64_t i = 0; i < n; ++i) pool->layout_ids[(size_t)i] = tensors[i].id;
        }
        return emit_plan(pool->plan, segs, n_segs, n_pages, fragmentation);
    });
}

extern "C" int apm_pack_tensors(apm_pool* pool, int state, const apm_tensor* tensors, int64_t n,
                                apm_segment* segs, int64_t* n_segs, int64_t* n_pages,
                                double* fragmentation, void* stream) {
    return apm::guarded([&]() -> int {
        if (!pool) return fail(APM_EINVAL, "NULL pool");
        if (pool->desc.device == APM_DEV_FILE) return fail(APM_EDEVICE, "pack / unpack work on GPU and HOST pools");
        if (!pool->stores(state)) return fail(APM_ERANGE, "pool does not store state class %d", state);
        int rc = check_list(tensors, n);
        if (rc != APM_OK) return rc;
        APM_HIP(hipSetDevice(pool->desc.hip_device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        if (!pool->has_layout) {
            Plan plan;
            rc = plan_of(pool, tensors, n, &plan);
            if (rc != APM_OK) return rc;
            rc = install_layout(pool, tensors, n, std::move(plan), s);
            if (rc != APM_OK) return rc;
        } else if (!same_layout(pool, tensors, n)) {
            return fail(APM_ESTATE, "tensor list does not match the pool's installed layout");
        }
        rc = emit_plan(pool->plan, segs, n_segs, n_pages, fragmentation);
        if (rc != APM_OK) return rc;
        return move_segments(pool, state, tensors, n, true, s);
    });
}

extern "C" int apm_unpack(apm_pool* pool, int state, const apm_tensor* dst, int64_t n, void* stream) {
    return apm::guarded([&]() -> int {
        if (!pool) return fail(APM_EINVAL, "NULL pool");
        if (pool->desc.device == APM_DEV_FILE) return fail(APM_EDEVICE, "pack / unpack work on GPU and HOST pools");
        if (!pool->stores(state)) return fail(APM_ERANGE, "pool does not store state class %d", state);
        int rc = check_list(dst, n);
        if (rc != APM_OK) return rc;
        if (!same_layout(pool, dst, n)) return fail(APM_ESTATE, "tensor list does not match the pool's installed layout");
        APM_HIP(hipSetDevice(pool->desc.hip_device));
        return move_segments(pool, state, dst, n, false, static_cast<hipStream_t>(stream));
    });
}

extern "C" int apm_page_copy_async(apm_pool* dst, int64_t dst_page, apm_pool* src, int64_t src_page,
                                   int64_t n_pages, int state, void* stream) {
    return apm::guarded([&]() -> int {
        if (!dst || !src) return fail(APM_EINVAL, "NULL pool");
        if (!dst->stores(state) || !src->stores(state)) return fail(APM_ERANGE, "state class %d is not stored by both pools", state);
        if (dst->desc.page_elems != src->desc.page_elems) return fail(APM_EINVAL, "pools have different page sizes");
        if (n_pages < 0) return fail(APM_EINVAL, "negative page count");
        if (dst_page < 0 || dst_page > dst->desc.n_pages || n_pages > dst->desc.n_pages - dst_page ||
            src_page < 0 || src_page > src->desc.n_pages || n_pages > src->desc.n_pages - src_page)
            return fail(APM_ERANGE, "page range out of bounds");
        if (n_pages == 0) return APM_OK;
        if (dst->desc.device == APM_DEV_FILE || src->desc.device == APM_DEV_FILE) {
            if (dst->desc.device == src->desc.device) return fail(APM_EDEVICE, "a FILE pool exchanges pages with HOST pools only");
            return file_page_copy(dst, dst_page, src, src_page, n_pages, state, static_cast<hipStream_t>(stream));
        }
        const size_t pb = (size_t)dst->desc.page_elems * (size_t)elem_bytes(state);
        char* d = static_cast<char*>(dst->base[state]) + (size_t)dst_page * pb;
        const char* s = static_cast<const char*>(src->base[state]) + (size_t)src_page * pb;
        if (dst == src && dst_page < src_page + n_pages && src_page < dst_page + n_pages && dst_page != src_page)
            return fail(APM_EINVAL, "overlapping page ranges");
        const bool dh = dst->desc.device == APM_DEV_HOST, sh = src->desc.device == APM_DEV_HOST;
        const hipMemcpyKind kind = sh ? (dh ? hipMemcpyHostToHost : hipMemcpyHostToDevice)
                                      : (dh ? hipMemcpyDeviceToHost : hipMemcpyDeviceToDevice);
        APM_HIP(hipSetDevice(dh ? src->desc.hip_device : dst->desc.hip_device));
        APM_HIP(hipMemcpyAsync(d, s, pb * (size_t)n_pages, kind, static_cast<hipStream_t>(stream)));
        return APM_OK;
    });
}

extern "C" int apm_pool_set_timing(apm_pool* pool, int enable) {
    return apm::guarded([&]() -> int {
        if (!pool) return fail(APM_EINVAL, "NULL pool");
        pool->timing = enable != 0;
        return APM_OK;
    });
}

extern "C" int apm_pool_read_timing(apm_pool* pool, double* ms, int64_t* launches) {
    return apm::guarded([&]() -> int {
        if (!pool || !ms || !launches) return fail(APM_EINVAL, "NULL argument");
        for (int k = 0; k < APM_N_KERNEL_CLASSES; ++k) {
            ms[k] = 0.0;
            launches[k] = 0;
        }
        int rc = APM_OK;
        for (auto& t : pool->timed) {
            float dt = 0.0f;
            hipError_t e = hipEventSynchronize(t.end);
            if (e == hipSuccess) e = hipEventElapsedTime(&dt, t.begin, t.end);
            if (e != hipSuccess) rc = fail(APM_EDEVICE, "reading a timing event failed: %s", hipGetErrorString(e));
            else {
                ms[t.cls] += (double)dt;
                launches[t.cls] += 1;
            }
            (void)hipEventDestroy(t.begin);
            (void)hipEventDestroy(t.end);
        }
        pool->timed.clear();
        return rc;
    });
}
