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
    return apm::guarded([&]() -> int {
        if (!n_segs) return apm::fail(APM_EINVAL, "n_segs is NULL");
        apm::Plan pl;
        int rc = apm::make_plan(page_elems, numels, n, &pl);
        if (rc != APM_OK) return rc;
        return apm::emit_plan(pl, segs, n_segs, n_pages, fragmentation);
    });
}

// ---- life-time based scheduling (Alg. 1, phase 1) ---------------------------------------------
//
// The schedule's movement tasks always cover a prefix of the page sequence (the layers' page lists
// laid end to end): tasks are only ever taken off the end and put back in sequence order.  So the
// planner's state is the length of that prefix, the number of pages resident once the schedule so
// far has run, and the task list with tombstones for the tasks taken off; every step is O(1).
extern "C" int apm_schedule_plan(const int64_t* layer_offsets, const int64_t* layer_pages,
                                 const int64_t* layer_bytes, int64_t n_layers,
                                 const int64_t* last_access, int64_t n_pages, int64_t page_bytes,
                                 int64_t gpu_memory_bytes, apm_task* tasks, int64_t* n_tasks,
                                 int64_t* peak_bytes) {
    return apm::guarded([&]() -> int {
        using apm::fail;
        if (!n_tasks) return fail(APM_EINVAL, "n_tasks is NULL");
        if (n_layers < 0 || n_pages < 0 || (n_layers > 0 && (!layer_offsets || !layer_bytes))) return fail(APM_EINVAL, "bad layer arrays");
        if (page_bytes <= 0 || gpu_memory_bytes < 0) return fail(APM_EINVAL, "page_bytes must be positive and gpu_memory_bytes non-negative");
        if (n_pages > 0 && page_bytes > (INT64_MAX >> 1) / n_pages) return fail(APM_EINVAL, "n_pages * page_bytes overflows");
        if (n_layers > INT32_MAX) return fail(APM_EINVAL, "too many layers");
        const int64_t P = n_layers > 0 ? layer_offsets[n_layers] : 0;
        if (n_layers > 0 && layer_offsets[0] != 0) return fail(APM_EINVAL, "layer_offsets[0] must be 0");
        if (P != n_pages) return fail(APM_EINVAL, "the layers list %lld pages, n_pages is %lld: every page belongs to exactly one layer", (long long)P, (long long)n_pages);
        if (P > 0 && !layer_pages) return fail(APM_EINVAL, "layer_pages is NULL");
        for (int64_t i = 0; i < n_layers; ++i)  // before anything is read through them
            if (layer_offsets[i + 1] < layer_offsets[i] || layer_offsets[i + 1] > P) return fail(APM_EINVAL, "layer_offsets must not decrease");
        std::vector<int32_t> owner((size_t)n_pages, -1);  // by page id
        for (int64_t i = 0; i < n_layers; ++i) {
            if (layer_bytes[i] < 0) return fail(APM_EINVAL, "layer_bytes[%lld] is negative", (long long)i);
            for (int64_t k = layer_offsets[i]; k < layer_offsets[i + 1]; ++k) {
                const int64_t p = layer_pages[k];
                if (p < 0 || p >= n_pages) return fail(APM_ERANGE, "layer %lld lists page %lld, out of range", (long long)i, (long long)p);
                if (owner[(size_t)p] >= 0) return fail(APM_EINVAL, "page %lld is listed twice", (long long)p);
                owner[(size_t)p] = (int32_t)i;
            }
        }
        std::vector<int64_t> released((size_t)n_layers, 0);  // pages whose last access is layer i
        for (int64_t p = 0; p < n_pages; ++p) {
            const int64_t la = last_access ? last_access[p] : owner[(size_t)p];
            if (la < owner[(size_t)p] || la >= n_layers) return fail(APM_EINVAL, "last_access[%lld] = %lld lies before the page's own layer or beyond the last layer", (long long)p, (long long)la);
            ++released[(size_t)la];
        }

        struct Slot { apm_task t; bool live; };
        std::vector<Slot> S;
        S.reserve((size_t)(2 * n_pages + n_layers));
        std::vector<int64_t> move_at;  // positions in S of the live movement tasks, in sequence order
        move_at.reserve((size_t)n_pages);
        int64_t resident = 0;
        auto push_move = [&](int64_t trigger) {  // the next page of the sequence
            const int64_t p = layer_pages[(int64_t)move_at.size()];
            move_at.push_back((int64_t)S.size());
            S.push_back({apm_task{APM_TASK_MOVE_TO_GPU, (int32_t)trigger, p}, true});
            ++resident;
        };
        auto available = [&]() { return gpu_memory_bytes - page_bytes * resident; };
        for (int64_t k = 0; k < n_pages; ++k) push_move(0);
        for (int64_t i = 0; i < n_layers; ++i) {
            // a page of this layer that is still deferred is fetched now
            while ((int64_t)move_at.size() < layer_offsets[i + 1]) push_move(i);
            while (available() < layer_bytes[i]) {
                // only pages of later layers can give way
                if ((int64_t)move_at.size() <= layer_offsets[i + 1])
                    return fail(APM_ENOMEM, "layer %lld does not fit: %lld resident pages of %lld bytes plus %lld bytes exceed %lld", (long long)i, (long long)resident, (long long)page_bytes, (long long)layer_bytes[i], (long long)gpu_memory_bytes);
                S[(size_t)move_at.back()].live = false;
                move_at.pop_back();
                --resident;
            }
            S.push_back({apm_task{APM_TASK_COMPUTE, (int32_t)i, i}, true});
            resident -= released[(size_t)i];
            while ((int64_t)move_at.size() < n_pages && available() > page_bytes) push_move(i);
        }
        const int64_t need_tasks = n_pages + n_layers;
        const int64_t cap = *n_tasks;
        *n_tasks = need_tasks;
        if (peak_bytes) {
            // measured on the finished schedule: a later layer may have taken back movements that
            // were still planned ahead of an earlier compute when that compute was appended
            int64_t on_gpu = 0, peak = 0;
            for (const Slot& sl : S) {
                if (!sl.live) continue;
                if (sl.t.op == APM_TASK_MOVE_TO_GPU) { ++on_gpu; continue; }
                const int64_t need = page_bytes * on_gpu + layer_bytes[sl.t.target];
                if (need > peak) peak = need;
                on_gpu -= released[(size_t)sl.t.target];
            }
            *peak_bytes = peak;
        }
        if (!tasks && cap == 0) return APM_OK;
        if (cap < need_tasks) return fail(APM_ERANGE, "task buffer holds %lld entries, %lld needed", (long long)cap, (long long)need_tasks);
        if (!tasks) return fail(APM_EINVAL, "tasks is NULL but *n_tasks is %lld", (long long)cap);
        int64_t n = 0;
        for (const Slot& sl : S)
            if (sl.live) tasks[n++] = sl.t;
        return APM_OK;
    });
}
