// Host side of the update: scalar preparation, page-list handling, the synchronous step and the
// one-step-stale (delayed) step.
#include <chrono>
#include <cmath>

#include "apm_internal.h"

namespace apm {

int prepare_hyper(const apm_hyper* h, int64_t step, AdamwLaunch* a) {
    if (!h) return fail(APM_EINVAL, "NULL hyper");
    if (step < 1) return fail(APM_EINVAL, "step must be >= 1 (got %lld): bias correction divides by 1 - beta^step", (long long)step);
    if (!(h->beta1 >= 0.0 && h->beta1 < 1.0) || !(h->beta2 >= 0.0 && h->beta2 < 1.0)) return fail(APM_EINVAL, "betas must lie in [0, 1)");
    if (!(h->eps >= 0.0) || !std::isfinite(h->lr) || !std::isfinite(h->weight_decay) || std::isnan(h->max_grad_norm)) return fail(APM_EINVAL, "bad hyper-parameter");
    if (h->skip_mode != APM_SKIP_NONE && h->skip_mode != APM_SKIP_UNTOUCHED) return fail(APM_EINVAL, "unknown skip_mode %d", h->skip_mode);
    // Every scalar is formed in double and rounded to fp32 exactly once: 1 - 0.999f evaluated in
    // fp32 would already be off by 1e-5 relative.
    const double bc1 = 1.0 - std::pow(h->beta1, (double)step);
    const double bc2 = 1.0 - std::pow(h->beta2, (double)step);
    a->b1 = (float)h->beta1;
    a->omb1 = (float)(1.0 - h->beta1);
    a->b2 = (float)h->beta2;
    a->omb2 = (float)(1.0 - h->beta2);
    a->inv_sqrt_bc2 = (float)(1.0 / std::sqrt(bc2));
    a->eps = (float)h->eps;
    a->step_size = (float)(h->lr / bc1);
    a->lr_wd = (float)(h->lr * h->weight_decay);
    a->max_norm = h->max_grad_norm > 0.0 ? h->max_grad_norm : 0.0;
    a->skip_mode = h->skip_mode;
    return APM_OK;
}

namespace {
// Checks a bf16 tensor list against the installed layout for the gather / scatter kernels.
int check_fused_list(const apm_pool* pool, const apm_tensor* t, int64_t n, const char* what) {
    if (!pool->has_layout || (int64_t)pool->layout_numels.size() != n) return fail(APM_ESTATE, "%s list does not match the pool's installed layout", what);
    for (int64_t i = 0; i < n; ++i) {
        if (t[i].numel != pool->layout_numels[(size_t)i]) return fail(APM_ESTATE, "%s list does not match the pool's installed layout", what);
        if (t[i].numel == 0) continue;
        if (t[i].dtype != APM_BF16) return fail(APM_EINVAL, "%s tensor %lld is not bf16", what, (long long)i);
        if (!t[i].data || (reinterpret_cast<uintptr_t>(t[i].data) & 15u)) return fail(APM_EINVAL, "%s tensor %lld: data must be a 16-byte aligned device pointer", what, (long long)i);
    }
    return APM_OK;
}
}  // namespace

int enqueue_step(apm_pool* pool, const int64_t* pages, int64_t n_pages, int64_t step,
                 const apm_hyper* hyper, const uint16_t* g16_override, float* grad_norm,
                 uint8_t* skip_mask, hipStream_t stream, const apm_tensor* grad_tensors,
                 const apm_tensor* p16_tensors, int64_t n_tensors) {
    if (!pool) return fail(APM_EINVAL, "NULL pool");
    if (pool->desc.device != APM_DEV_GPU) return fail(APM_EDEVICE, "the update runs on GPU pools only");
    for (int st = 0; st < APM_N_STATES; ++st) {
        if (st == APM_G16 && (g16_override || grad_tensors)) continue;
        if (st == APM_P16 && p16_tensors) continue;
        if (!pool->stores(st)) return fail(APM_ESTATE, "pool does not store state class %d", st);
    }
    if (grad_tensors) {
        int rc0 = check_fused_list(pool, grad_tensors, n_tensors, "gradient");
        if (rc0 != APM_OK) return rc0;
    }
    if (p16_tensors) {
        int rc0 = check_fused_list(pool, p16_tensors, n_tensors, "bf16 parameter");
        if (rc0 != APM_OK) return rc0;
    }
    if (n_pages < 0 || n_pages > pool->desc.n_pages) return fail(APM_ERANGE, "page count %lld out of range", (long long)n_pages);
    AdamwLaunch L{};
    int rc = prepare_hyper(hyper, step, &L);
    if (rc != APM_OK) return rc;
    if (n_pages == 0) return APM_OK;
    APM_HIP(hipSetDevice(pool->desc.hip_device));

    // List positions are grouped into extent classes (largest extents first, the caller's order
    // kept inside a class).  order[pos] = the caller's index of the page launched at position pos.
    const int64_t E = pool->desc.page_elems;
    const int64_t in_use = pool->has_layout ? (int64_t)pool->plan.pages.size() : 0;
    auto page_at = [&](int64_t k) { return pages ? pages[k] : k; };
    auto used_of = [&](int64_t page) { return page < in_use ? pool->plan.pages[(size_t)page].used : (int64_t)0; };
    if (pages) {
        // Two workgroups updating one page at once would race: a listed page is listed once.
        std::vector<uint8_t> seen((size_t)pool->desc.n_pages, 0);
        for (int64_t k = 0; k < n_pages; ++k) {
            if (pages[k] < 0 || pages[k] >= pool->desc.n_pages) return fail(APM_ERANGE, "pages[%lld] = %lld out of range [0, %lld)", (long long)k, (long long)pages[k], (long long)pool->desc.n_pages);
            if (seen[(size_t)pages[k]]) return fail(APM_EINVAL, "pages[%lld] = %lld is listed twice", (long long)k, (long long)pages[k]);
            seen[(size_t)pages[k]] = 1;
        }
    }
    if (grad_tensors || p16_tensors) {  // the tensors cover the pages of the layout and no others
        if (!pages && n_pages > in_use) return fail(APM_ERANGE, "page count %lld exceeds the %lld pages in use", (long long)n_pages, (long long)in_use);
        if (pages)
            for (int64_t k = 0; k < n_pages; ++k)
                if (pages[k] >= in_use) return fail(APM_ERANGE, "pages[%lld] = %lld is not in use by the layout", (long long)k, (long long)pages[k]);
    }
    auto class_of = [&](int64_t used) { return used * 4 > E ? 0 : used * 32 > E ? 1 : used * 512 > E ? 2 : 3; };
    int64_t cnt[kMaxExtentClasses] = {}, mx[kMaxExtentClasses] = {};
    for (int64_t k = 0; k < n_pages; ++k) {
        const int64_t u = used_of(page_at(k));
        const int c = class_of(u);
        ++cnt[c];
        if (u > mx[c]) mx[c] = u;
    }
    // A class is worth its extra launches only if it saves enough idle workgroups (counted in
    // 1024-element update slices); otherwise it is folded into the next larger one.
    int into[kMaxExtentClasses];
    for (int c = 0; c < kMaxExtentClasses; ++c) into[c] = c;
    constexpr int64_t kUpdateSpan = 1024, kWorthWorkgroups = 16384;
    for (int c = kMaxExtentClasses - 1; c > 0; --c) {
        if (cnt[c] == 0) continue;
        int j = c - 1;
        while (j > 0 && cnt[j] == 0) --j;
        if (cnt[j] == 0) continue;
        if (cnt[c] * ((mx[j] - mx[c]) / kUpdateSpan) < kWorthWorkgroups) {
            for (int q = c; q < kMaxExtentClasses; ++q) if (into[q] == c) into[q] = j;
            cnt[j] += cnt[c];
            cnt[c] = 0;
        }
    }
    int64_t begin[kMaxExtentClasses];
    for (int64_t c = 0, at = 0; c < kMaxExtentClasses; ++c) {
        begin[c] = at;
        if (cnt[c] > 0) L.cls[L.n_cls++] = ExtentClass{at, cnt[c], mx[c]};
        at += cnt[c];
    }
    std::vector<int64_t> order((size_t)n_pages);
    bool identity = true;
    {
        int64_t fill[kMaxExtentClasses];
        for (int c = 0; c < kMaxExtentClasses; ++c) fill[c] = begin[c];
        for (int64_t k = 0; k < n_pages; ++k) {
            const int c = into[class_of(used_of(page_at(k)))];
            const int64_t pos = fill[c]++;
            order[(size_t)pos] = k;
            if (pos != k) identity = false;
        }
    }

    // A list that is an ascending run launched in the caller's order needs no indirection;
    // anything else is staged to the device: page indices, then the output indices.
    const int64_t first = page_at(0);
    bool run = identity;
    for (int64_t k = 0; run && k < n_pages; ++k)
        if (page_at(k) != first + k) run = false;
    int ring_slots[2], n_ring_slots = 0;  // sealed once the kernels that read them are enqueued
    const int64_t* d_list = nullptr;
    if (!run) {
        const size_t list_bytes = (size_t)n_pages * sizeof(int64_t);
        const size_t bytes = list_bytes + (size_t)n_pages * sizeof(int32_t);
        int slot;
        rc = pool->ring.acquire(bytes, &slot);
        if (rc != APM_OK) return rc;
        int64_t* h = static_cast<int64_t*>(pool->ring.h[slot]);
        int32_t* ho = reinterpret_cast<int32_t*>(static_cast<char*>(pool->ring.h[slot]) + list_bytes);
        for (int64_t k = 0; k < n_pages; ++k) {
            h[k] = page_at(order[(size_t)k]);
            ho[k] = (int32_t)order[(size_t)k];
        }
        rc = pool->ring.commit(slot, bytes, stream);
        if (rc != APM_OK) return rc;
        ring_slots[n_ring_slots++] = slot;
        d_list = static_cast<const int64_t*>(pool->ring.d[slot]);
        if (!identity) L.out_index = reinterpret_cast<const int32_t*>(static_cast<const char*>(pool->ring.d[slot]) + list_bytes);
    }

    if (grad_tensors || p16_tensors) {
        // One PageSegs entry per list position, rebuilt per call: the tensors are caller-owned and
        // their addresses may change from step to step.
        const size_t n_in_use = pool->plan.pages.size();
        std::vector<PageSegs> by_page(n_in_use);
        std::vector<uint8_t> filled(n_in_use, 0);
        for (const apm_segment& sg : pool->plan.segs) {  // a page's tenants appear in offset order
            PageSegs& e = by_page[(size_t)sg.page];
            const int k = filled[(size_t)sg.page]++;
            e.off[k] = (int32_t)sg.page_off;
            e.n[k] = (int32_t)sg.n;
            if (grad_tensors) e.g[k] = static_cast<const uint16_t*>(grad_tensors[sg.tensor].data) + sg.tensor_off;
            if (p16_tensors) e.q[k] = static_cast<uint16_t*>(p16_tensors[sg.tensor].data) + sg.tensor_off;
        }
        int slot;
        rc = pool->ring.acquire((size_t)n_pages * sizeof(PageSegs), &slot);
        if (rc != APM_OK) return rc;
        PageSegs* h = static_cast<PageSegs*>(pool->ring.h[slot]);
        for (int64_t k = 0; k < n_pages; ++k) h[k] = by_page[(size_t)page_at(order[(size_t)k])];
        rc = pool->ring.commit(slot, (size_t)n_pages * sizeof(PageSegs), stream);
        if (rc != APM_OK) return rc;
        ring_slots[n_ring_slots++] = slot;
        L.segs = static_cast<const PageSegs*>(pool->ring.d[slot]);
        L.gather = grad_tensors != nullptr;
        L.scatter = p16_tensors != nullptr;
    }
    L.p32 = static_cast<float*>(pool->base[APM_P32]);
    L.m32 = static_cast<float*>(pool->base[APM_M32]);
    L.v32 = static_cast<float*>(pool->base[APM_V32]);
    L.g16 = g16_override ? g16_override : static_cast<const uint16_t*>(pool->base[APM_G16]);
    L.p16 = static_cast<uint16_t*>(pool->base[APM_P16]);
    L.used = pool->d_used;
    L.state_pages = L.grad_pages = d_list;
    L.state_first = L.grad_first = first;
    L.n_listed = n_pages;
    L.E = E;
    L.S = pool->S;
    L.grad_norm = grad_norm;
    L.skip_mask = skip_mask;
    const bool need_reduce = grad_norm || skip_mask || L.max_norm > 0.0 || L.skip_mode != APM_SKIP_NONE;
    rc = ensure_scratch(pool);
    if (rc != APM_OK) return rc;
    L.meta = pool->d_meta;
    if (need_reduce) {
        L.partials = pool->d_partials;
        L.nzflags = pool->d_nzflags;
        ScopedTiming t(pool, APM_K_REDUCE, stream);
        APM_HIP(launch_grad_reduce(L, stream));
    } else {
        APM_HIP(launch_prepare(L, stream));
    }
    {
        ScopedTiming t(pool, APM_K_UPDATE, stream);
        APM_HIP(launch_adamw(L, stream));
    }
    for (int k = 0; k < n_ring_slots; ++k) {
        rc = pool->ring.seal(ring_slots[k], stream);
        if (rc != APM_OK) return rc;
    }
    return APM_OK;
}

namespace {
// Spins for `ticks` of the constant-rate device clock; the iteration cap makes it end regardless.
__global__ void apm_spin_kernel(long long ticks, int max_iters) {
    const long long t0 = wall_clock64();
    for (int i = 0; i < max_iters; ++i) {
        if (wall_clock64() - t0 >= ticks) break;
        __builtin_amdgcn_s_sleep(32);
    }
}
}  // namespace

int streams_overlap(hipStream_t a, hipStream_t b, bool* out) {
    int dev = 0, khz = 0;
    APM_HIP(hipGetDevice(&dev));
    APM_HIP(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) khz = 100000;
    constexpr double kSpinMs = 0.5;
    const long long ticks = (long long)(kSpinMs * khz);
    const int cap = 20000;  // >= 1 us per iteration: the kernel ends after some tens of ms at most
    auto both = [&](long long t, double* ms) -> int {
        APM_HIP(hipStreamSynchronize(a));
        APM_HIP(hipStreamSynchronize(b));
        const auto t0 = std::chrono::steady_clock::now();
        hipLaunchKernelGGL(apm_spin_kernel, dim3(1), dim3(1), 0, a, t, cap);
        hipLaunchKernelGGL(apm_spin_kernel, dim3(1), dim3(1), 0, b, t, cap);
        APM_HIP(hipGetLastError());
        APM_HIP(hipStreamSynchronize(a));
        APM_HIP(hipStreamSynchronize(b));
        *ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
        return APM_OK;
    };
    double warm, ms1, ms2;
    int rc = both(0, &warm);  // loads the kernel
    if (rc == APM_OK) rc = both(ticks, &ms1);
    if (rc == APM_OK) rc = both(ticks, &ms2);
    if (rc != APM_OK) return rc;
    const double ms = ms1 < ms2 ? ms1 : ms2;
    *out = ms < 1.6 * kSpinMs;  // side by side: ~0.5 ms; one after the other: ~1 ms
    return APM_OK;
}

int make_overlapping_stream(hipStream_t with, hipStream_t* out, bool* overlaps, const hipStream_t* also) {
    constexpr int kTries = 8;
    hipStream_t cand[kTries] = {};
    int n = 0, pick = -1;
    int rc = APM_OK;
    // Rejected candidates stay alive until the choice is made: a destroyed stream's queue slot
    // would be handed straight to the next one created.
    for (; n < kTries && pick < 0; ++n) {
        if (hipStreamCreateWithFlags(&cand[n], hipStreamNonBlocking) != hipSuccess) {
            (void)hipGetLastError();
            rc = fail(APM_EDEVICE, "creating a stream failed");
            break;
        }
        bool ok = false;
        rc = streams_overlap(with, cand[n], &ok);
        if (rc == APM_OK && ok && also) rc = streams_overlap(*also, cand[n], &ok);
        if (rc != APM_OK) { ++n; break; }
        if (ok) pick = n;
    }
    if (rc == APM_OK && pick < 0 && n > 0) pick = n - 1;
    for (int k = 0; k < n; ++k)
        if (k != pick && cand[k]) (void)hipStreamDestroy(cand[k]);
    if (rc != APM_OK) {
        if (pick >= 0 && cand[pick]) (void)hipStreamDestroy(cand[pick]);
        return rc;
    }
    *out = cand[pick];
    bool ok = false;
    rc = streams_overlap(with, cand[pick], &ok);
    if (rc == APM_OK && ok && also) rc = streams_overlap(*also, cand[pick], &ok);
    if (overlaps) *overlaps = rc == APM_OK && ok;
    return APM_OK;
}

int ensure_delayed(apm_pool* pool, hipStream_t caller, bool probe) {
    if (pool->upd_stream) return APM_OK;
    const size_t bytes = (size_t)pool->desc.n_pages * (size_t)pool->desc.page_elems * 2u;
    for (int k = 0; k < 2; ++k) {
        if (pool->gbuf[k]) continue;  // kept from an attempt that failed further down
        hipError_t e = hipMalloc((void**)&pool->gbuf[k], bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            for (int j = 0; j < 2; ++j) {
                if (pool->gbuf[j]) (void)hipFree(pool->gbuf[j]);
                pool->gbuf[j] = nullptr;
            }
            return fail(APM_ENOMEM, "allocating the %zu-byte buffered-gradient halves failed: %s", bytes, hipGetErrorString(e));
        }
    }
    // Zero once: a producer that fills a half in place writes its tensors' elements only, and the
    // alignment gaps inside a page's used extent are read as gradient.
    for (int k = 0; k < 2; ++k) APM_HIP(hipMemset(pool->gbuf[k], 0, bytes));
    for (int k = 0; k < 2; ++k) {
        if (!pool->ev_staged[k]) APM_HIP(hipEventCreateWithFlags(&pool->ev_staged[k], hipEventDisableTiming));
        if (!pool->ev_applied[k]) APM_HIP(hipEventCreateWithFlags(&pool->ev_applied[k], hipEventDisableTiming));
    }
    if (!pool->ev_flush) APM_HIP(hipEventCreateWithFlags(&pool->ev_flush, hipEventDisableTiming));
    // The update stream must run beside the producer's stream, which is the point of the
    // one-step-stale form; which streams do is measured, once, here.
    if (probe) return make_overlapping_stream(caller, &pool->upd_stream, &pool->upd_overlaps);
    APM_HIP(hipStreamCreateWithFlags(&pool->upd_stream, hipStreamNonBlocking));
    return APM_OK;
}

// Applies the buffered gradient (half `cur`) on the update stream.
static int apply_buffered(apm_pool* pool, const DelayedApply& apply) {
    const int k = pool->cur;
    APM_HIP(hipStreamWaitEvent(pool->upd_stream, pool->ev_staged[k], 0));
    int rc = apply(pool->gbuf[k], pool->applied + 1, pool->upd_stream,
                   pool->buf_pages_null ? nullptr : pool->buf_pages.data(), pool->buf_n_pages, &pool->buf_hyper);
    if (rc != APM_OK) return rc;
    pool->applied += 1;
    APM_HIP(hipEventRecord(pool->ev_applied[k], pool->upd_stream));
    pool->applied_valid[k] = true;
    return APM_OK;
}

int delayed_call(apm_pool* pool, const int64_t* pages, int64_t n_pages, const void* new_g16,
                 const apm_hyper* hyper, hipStream_t s, const DelayedApply& apply) {
    APM_HIP(hipSetDevice(pool->desc.hip_device));
    int rc = ensure_delayed(pool, s, true);
    if (rc != APM_OK) return rc;
    if (pool->buffered) {
        rc = apply_buffered(pool, apply);
        if (rc != APM_OK) return rc;
        pool->buffered = false;
    }
    if (!new_g16) {  // flush: the caller's stream joins the update stream
        APM_HIP(hipEventRecord(pool->ev_flush, pool->upd_stream));
        APM_HIP(hipStreamWaitEvent(s, pool->ev_flush, 0));
        return APM_OK;
    }
    // Stage the new gradient into the other half; that half was last read by the update enqueued
    // two calls ago, which must have finished before it is overwritten.
    const int nxt = pool->cur ^ 1;
    const size_t pb = (size_t)pool->desc.page_elems * 2u;
    // The gradient travels with the list and the hyper-parameters of this call (copied before
    // anything is enqueued: an allocation failure leaves the pool as it was).
    std::vector<int64_t> list_copy;
    if (pages) list_copy.assign(pages, pages + n_pages);
    const char* src = static_cast<const char*>(new_g16);
    char* dst = reinterpret_cast<char*>(pool->gbuf[nxt]);
    // A producer that wrote its gradient straight into the half handed out by
    // apm_delayed_grad_buffer has already staged it (and waited for the half to be free there).
    const bool in_place = src == dst;
    if (!in_place && pool->applied_valid[nxt]) APM_HIP(hipStreamWaitEvent(s, pool->ev_applied[nxt], 0));
    int64_t k = in_place ? n_pages : 0;
    while (k < n_pages) {  // one copy per run of consecutive pages
        const int64_t p0 = pages ? pages[k] : k;
        int64_t len = 1;
        while (k + len < n_pages && (pages ? pages[k + len] : k + len) == p0 + len) ++len;
        APM_HIP(hipMemcpyAsync(dst + (size_t)p0 * pb, src + (size_t)p0 * pb, pb * (size_t)len, hipMemcpyDeviceToDevice, s));
        k += len;
    }
    APM_HIP(hipEventRecord(pool->ev_staged[nxt], s));
    pool->buf_hyper = *hyper;
    pool->buf_pages.swap(list_copy);
    pool->buf_pages_null = pages == nullptr;
    pool->buf_n_pages = n_pages;
    pool->cur = nxt;
    pool->buffered = true;
    return APM_OK;
}

}  // namespace apm

using namespace apm;

extern "C" int apm_page_adamw_step(apm_pool* pool, const int64_t* pages, int64_t n_pages,
                                   int64_t step, const apm_hyper* hyper, float* grad_norm,
                                   uint8_t* skip_mask, void* stream) {
    return apm::guarded([&]() -> int {
        return enqueue_step(pool, pages, n_pages, step, hyper, nullptr, grad_norm, skip_mask,
                            static_cast<hipStream_t>(stream));
    });
}

extern "C" int apm_page_adamw_step_fused(apm_pool* pool, const int64_t* pages, int64_t n_pages,
                                         int64_t step, const apm_hyper* hyper,
                                         const apm_tensor* grad_tensors,
                                         const apm_tensor* p16_tensors, int64_t n_tensors,
                                         float* grad_norm, uint8_t* skip_mask, void* stream) {
    return apm::guarded([&]() -> int {
        if (!grad_tensors && !p16_tensors) return fail(APM_EINVAL, "neither a gradient nor a parameter tensor list was given");
        if (n_tensors < 0) return fail(APM_EINVAL, "negative tensor count");
        return enqueue_step(pool, pages, n_pages, step, hyper, nullptr, grad_norm, skip_mask,
                            static_cast<hipStream_t>(stream), grad_tensors, p16_tensors, n_tensors);
    });
}

extern "C" int apm_step_delayed(apm_pool* pool, const int64_t* pages, int64_t n_pages,
                                const void* new_g16, const apm_hyper* hyper, void* stream) {
    return apm::guarded([&]() -> int {
        if (!pool) return fail(APM_EINVAL, "NULL pool");
        if (pool->desc.device != APM_DEV_GPU) return fail(APM_EDEVICE, "the update runs on GPU pools only");
        if (n_pages < 0 || n_pages > pool->desc.n_pages) return fail(APM_ERANGE, "page count %lld out of range", (long long)n_pages);
        AdamwLaunch probe{};
        int rc = prepare_hyper(hyper, 1, &probe);  // validate before any state changes
        if (rc != APM_OK) return rc;
        if (pages)
            for (int64_t k = 0; k < n_pages; ++k)
                if (pages[k] < 0 || pages[k] >= pool->desc.n_pages) return fail(APM_ERANGE, "pages[%lld] out of range", (long long)k);
        return delayed_call(pool, pages, n_pages, new_g16, hyper, static_cast<hipStream_t>(stream),
                            [&](const uint16_t* g16, int64_t step, hipStream_t upd, const int64_t* b_pages,
                                int64_t b_n, const apm_hyper* b_hyper) {
                                return enqueue_step(pool, b_pages, b_n, step, b_hyper, g16, pool->delayed_norm,
                                                    pool->delayed_skip, upd);
                            });
    });
}

extern "C" int apm_delayed_accumulate(apm_pool* pool, const int64_t* pages, int64_t n_pages,
                                      const void* g16, void* stream) {
    return apm::guarded([&]() -> int {
        if (!pool || !g16) return fail(APM_EINVAL, "NULL argument");
        if (pool->desc.device != APM_DEV_GPU) return fail(APM_EDEVICE, "GPU pools only");
        if (!pool->buffered) return fail(APM_ESTATE, "no gradient is being collected: call apm_step_delayed with a gradient first");
        if (n_pages < 0 || n_pages > pool->desc.n_pages) return fail(APM_ERANGE, "page count %lld out of range", (long long)n_pages);
        if (n_pages == 0) return APM_OK;
        APM_HIP(hipSetDevice(pool->desc.hip_device));
        hipStream_t s = static_cast<hipStream_t>(stream);
        int64_t first = 0;
        bool run = true;
        if (pages) {
            first = pages[0];
            for (int64_t k = 0; k < n_pages; ++k) {
                if (pages[k] < 0 || pages[k] >= pool->desc.n_pages) return fail(APM_ERANGE, "pages[%lld] out of range", (long long)k);
                if (pages[k] != first + k) run = false;
            }
        }
        const int64_t* d_list = nullptr;
        int slot = -1;
        if (!run) {
            int rc = pool->ring.acquire((size_t)n_pages * sizeof(int64_t), &slot);
            if (rc != APM_OK) return rc;
            int64_t* h = static_cast<int64_t*>(pool->ring.h[slot]);
            for (int64_t k = 0; k < n_pages; ++k) h[k] = pages[k];
            rc = pool->ring.commit(slot, (size_t)n_pages * sizeof(int64_t), s);
            if (rc != APM_OK) return rc;
            d_list = static_cast<const int64_t*>(pool->ring.d[slot]);
        }
        // The collecting half was staged on the producer's stream; the sum is ordered after it there,
        // and the "staged" event moves behind the sum so that the update sees the accumulated values.
        const int k = pool->cur;
        APM_HIP(hipStreamWaitEvent(s, pool->ev_staged[k], 0));
        APM_HIP(launch_grad_accum(pool->gbuf[k], static_cast<const uint16_t*>(g16), pool->d_used, d_list, first,
                                  n_pages, pool->desc.page_elems, s));
        APM_HIP(hipEventRecord(pool->ev_staged[k], s));
        if (slot >= 0) return pool->ring.seal(slot, s);
        return APM_OK;
    });
}

extern "C" void* apm_delayed_grad_buffer(apm_pool* pool, void* stream) {
    if (!pool || pool->desc.device != APM_DEV_GPU) {
        fail(APM_EINVAL, "NULL or non-GPU pool");
        return nullptr;
    }
    if (hipSetDevice(pool->desc.hip_device) != hipSuccess ||
        ensure_delayed(pool, static_cast<hipStream_t>(stream), true) != APM_OK) return nullptr;
    const int nxt = pool->cur ^ 1;
    if (pool->applied_valid[nxt] &&
        hipStreamWaitEvent(static_cast<hipStream_t>(stream), pool->ev_applied[nxt], 0) != hipSuccess) {
        fail(APM_EDEVICE, "hipStreamWaitEvent failed");
        return nullptr;
    }
    return pool->gbuf[nxt];
}

extern "C" int64_t apm_delayed_applied(const apm_pool* pool) { return pool ? pool->applied : 0; }

extern "C" int apm_delayed_set_outputs(apm_pool* pool, float* grad_norm, uint8_t* skip_mask) {
    return apm::guarded([&]() -> int {
        if (!pool) return fail(APM_EINVAL, "NULL pool");
        pool->delayed_norm = grad_norm;
        pool->delayed_skip = skip_mask;
        return APM_OK;
    });
}
