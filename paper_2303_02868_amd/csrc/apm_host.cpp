// Host-only parts: thread-local error text and the packing plan.  No HIP call in this file.
#include <cstdarg>
#include <cstdio>

#include "apm_internal.h"

namespace {
thread_local char g_err[512] = "";
}

namespace apm {

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// Layout rule of Sec. 4.1 as read by this library: at most two tenants per page, a tensor
// smaller than a page alone in a page, larger tensors chained through an "open" partly filled page.
int make_plan(int64_t E, const int64_t* numels, int64_t n, Plan* out) {
    if (E <= 0 || E % kAlign != 0) return fail(APM_EINVAL, "page_elems must be a positive multiple of %lld", (long long)kAlign);
    if (n < 0 || (n > 0 && !numels)) return fail(APM_EINVAL, "bad tensor list");
    Plan& pl = *out;
    pl = Plan();
    pl.E = E;
    int64_t open_page = -1;
    auto place = [&](int64_t t, int64_t t_off, int64_t page, int64_t p_off, int64_t cnt) {
        PageEntry& e = pl.pages[page];
        e.tensor[e.n_tensors] = t;
        e.tensor_elems[e.n_tensors] = cnt;
        e.n_tensors += 1;
        e.used = p_off + cnt;
        pl.segs.push_back(apm_segment{t, t_off, page, p_off, cnt});
    };
    for (int64_t t = 0; t < n; ++t) {
        const int64_t numel = numels[t];
        if (numel < 0) return fail(APM_EINVAL, "tensor %lld has negative numel", (long long)t);
        pl.total += numel;
        if (numel == 0) continue;
        if (numel < E) {  // small tensor: a page of its own, never shared
            pl.pages.emplace_back();
            place(t, 0, (int64_t)pl.pages.size() - 1, 0, numel);
            continue;
        }
        int64_t done = 0;
        if (open_page >= 0) {
            const int64_t start = (pl.pages[open_page].used + kAlign - 1) / kAlign * kAlign;
            if (start < E) {
                place(t, 0, open_page, start, E - start);
                done = E - start;
            }
            open_page = -1;
        }
        while (done < numel) {
            const int64_t cnt = numel - done < E ? numel - done : E;
            pl.pages.emplace_back();
            place(t, done, (int64_t)pl.pages.size() - 1, 0, cnt);
            done += cnt;
            if (cnt < E) open_page = (int64_t)pl.pages.size() - 1;
        }
    }
    return APM_OK;
}

int emit_plan(const Plan& pl, apm_segment* segs, int64_t* n_segs, int64_t* n_pages,
              double* fragmentation) {
    const int64_t need = (int64_t)pl.segs.size();
    if (n_pages) *n_pages = (int64_t)pl.pages.size();
    if (fragmentation)
        *fragmentation = pl.pages.empty() ? 0.0
                                          : 1.0 - (double)pl.total / ((double)pl.pages.size() * (double)pl.E);
    if (n_segs) {
        const int64_t cap = *n_segs;
        *n_segs = need;
        if (segs || cap != 0) {
            if (cap < need) return fail(APM_ENOMEM, "segment buffer holds %lld entries, %lld needed", (long long)cap, (long long)need);
            if (!segs) return fail(APM_EINVAL, "segs is NULL but *n_segs is %lld", (long long)cap);
            for (int64_t i = 0; i < need; ++i) segs[i] = pl.segs[i];
        }
    }
    return APM_OK;
}

}  // namespace apm

extern "C" const char* apm_last_error(void) { return g_err; }

extern "C" int apm_pack_plan(int64_t page_elems, const int64_t* numels, int64_t n,
                             apm_segment* segs, int64_t* n_segs, int64_t* n_pages,
                             double* fragmentation) {
    if (!n_segs) return apm::fail(APM_EINVAL, "n_segs is NULL");
    apm::Plan pl;
    int rc = apm::make_plan(page_elems, numels, n, &pl);
    if (rc != APM_OK) return rc;
    return apm::emit_plan(pl, segs, n_segs, n_pages, fragmentation);
}
