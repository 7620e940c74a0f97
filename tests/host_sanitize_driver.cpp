// Drives the library's host-only entry points (packing plan, Alg. 1 planner) with random and
// malformed inputs.  Built with AddressSanitizer + UBSan by tests/test_host_sanitizers.py: a
// memory error or undefined behaviour in the host logic aborts the run.  The checks in here are
// structural only (bounds, counts, coverage); values are checked against the oracle elsewhere.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "apm.h"

namespace {

struct Rng {  // splitmix64
    uint64_t s;
    uint64_t next() {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    int64_t below(int64_t n) { return n <= 0 ? 0 : (int64_t)(next() % (uint64_t)n); }
};

[[noreturn]] void die(const char* what, long long a = 0, long long b = 0) {
    std::fprintf(stderr, "driver check failed: %s (%lld, %lld); last error: %s\n", what, a, b, apm_last_error());
    std::exit(1);
}

void pack_case(Rng& r) {
    const int64_t E = 8 * (1 + r.below(64));
    const int64_t n = r.below(40);
    std::vector<int64_t> numels((size_t)n);
    int64_t total = 0;
    for (auto& x : numels) {
        switch (r.below(4)) {
            case 0: x = r.below(E); break;            // smaller than a page (0 included)
            case 1: x = E * (1 + r.below(3)); break;  // whole pages
            default: x = r.below(5 * E); break;
        }
        total += x;
    }
    int64_t n_segs = 0, n_pages = -1;
    double frag = -1;
    if (apm_pack_plan(E, numels.data(), n, nullptr, &n_segs, &n_pages, &frag) != APM_OK) die("pack query");
    if (n_segs < 0 || n_pages < 0 || frag < 0.0 || frag > 1.0) die("pack query outputs", n_segs, n_pages);
    // a buffer one entry short must be refused without being written past its end
    if (n_segs > 0) {
        std::vector<apm_segment> shorter((size_t)(n_segs - 1));
        int64_t cap = n_segs - 1;
        apm_segment dummy;
        int rc = apm_pack_plan(E, numels.data(), n, cap ? shorter.data() : &dummy, &cap, nullptr, nullptr);
        if (n_segs - 1 > 0 && rc != APM_ENOMEM) die("short buffer accepted", rc);
        if (n_segs - 1 > 0 && cap != n_segs) die("needed count not reported", cap, n_segs);
    }
    std::vector<apm_segment> segs((size_t)n_segs);
    int64_t cap = n_segs;
    if (apm_pack_plan(E, numels.data(), n, segs.data(), &cap, &n_pages, &frag) != APM_OK) die("pack fill");
    std::vector<int64_t> covered((size_t)n, 0), tenants((size_t)n_pages, 0), fill((size_t)n_pages, 0);
    for (const apm_segment& s : segs) {
        if (s.tensor < 0 || s.tensor >= n || s.page < 0 || s.page >= n_pages) die("segment ids", s.tensor, s.page);
        if (s.n <= 0 || s.page_off < 0 || s.page_off % 8 != 0 || s.page_off + s.n > E) die("segment extent", s.page_off, s.n);
        if (s.tensor_off != covered[(size_t)s.tensor]) die("tensor not covered in order", s.tensor, s.tensor_off);
        if (s.page_off < fill[(size_t)s.page]) die("segments overlap in a page", s.page, s.page_off);
        covered[(size_t)s.tensor] += s.n;
        fill[(size_t)s.page] = s.page_off + s.n;
        if (++tenants[(size_t)s.page] > 2) die("more than two tenants", s.page);
    }
    for (int64_t t = 0; t < n; ++t)
        if (covered[(size_t)t] != numels[(size_t)t]) die("tensor not fully placed", t, covered[(size_t)t]);
    for (int64_t p = 0; p < n_pages; ++p)
        if (tenants[(size_t)p] == 0) die("empty page in the plan", p);
    (void)total;
}

void pack_errors() {
    int64_t n_segs = 0;
    int64_t one = 5, neg = -1;
    if (apm_pack_plan(0, &one, 1, nullptr, &n_segs, nullptr, nullptr) != APM_EINVAL) die("E = 0 accepted");
    if (apm_pack_plan(12, &one, 1, nullptr, &n_segs, nullptr, nullptr) != APM_EINVAL) die("E = 12 accepted");
    if (apm_pack_plan(8, &neg, 1, nullptr, &n_segs, nullptr, nullptr) != APM_EINVAL) die("negative numel accepted");
    if (apm_pack_plan(8, nullptr, 1, nullptr, &n_segs, nullptr, nullptr) != APM_EINVAL) die("NULL numels accepted");
    if (apm_pack_plan(8, &one, 1, nullptr, nullptr, nullptr, nullptr) != APM_EINVAL) die("NULL n_segs accepted");
    if (apm_pack_plan(8, nullptr, 0, nullptr, &n_segs, nullptr, nullptr) != APM_OK || n_segs != 0) die("empty list");
}

void plan_case(Rng& r) {
    const int64_t L = r.below(12);
    std::vector<int64_t> off((size_t)L + 1, 0), bytes((size_t)L);
    for (int64_t i = 0; i < L; ++i) {
        off[(size_t)i + 1] = off[(size_t)i] + r.below(6);
        bytes[(size_t)i] = r.below(5000);
    }
    const int64_t P = off[(size_t)L];
    std::vector<int64_t> pages((size_t)P), owner((size_t)P, 0), last((size_t)P);
    for (int64_t k = 0; k < P; ++k) pages[(size_t)k] = k;
    for (int64_t k = P - 1; k > 0; --k) std::swap(pages[(size_t)k], pages[(size_t)r.below(k + 1)]);
    for (int64_t i = 0; i < L; ++i)
        for (int64_t k = off[(size_t)i]; k < off[(size_t)i + 1]; ++k) owner[(size_t)pages[(size_t)k]] = i;
    for (int64_t p = 0; p < P; ++p) last[(size_t)p] = owner[(size_t)p] + r.below(L - owner[(size_t)p]);
    const int64_t page_bytes = 1 + r.below(2000);
    const int64_t budget = r.below(page_bytes * (P + 2) + 6000);
    const bool with_last = r.below(3) != 0;
    // what is damaged in this case, if anything
    const int damage = (int)r.below(8);
    int expect_bad = 0;
    if (P > 0 && L > 0) {
        if (damage == 1) { pages[(size_t)r.below(P)] = P + r.below(3); expect_bad = 1; }
        else if (damage == 2 && P > 1) { pages[0] = pages[1]; expect_bad = 1; }
        else if (damage == 3 && with_last) { last[(size_t)r.below(P)] = L + r.below(2); expect_bad = 1; }
        else if (damage == 4) { bytes[(size_t)r.below(L)] = -1; expect_bad = 1; }
    }
    int64_t n_tasks = 0, peak = -1;
    int rc = apm_schedule_plan(off.data(), pages.data(), bytes.data(), L, with_last ? last.data() : nullptr, P,
                               page_bytes, budget, nullptr, &n_tasks, &peak);
    if (expect_bad) {
        if (rc == APM_OK) die("damaged trace accepted", damage);
        return;
    }
    if (rc == APM_ENOMEM) return;
    if (rc != APM_OK) die("plan query", rc);
    if (n_tasks != P + L) die("task count", n_tasks, P + L);
    if (peak < 0 || peak > budget) die("peak beyond the budget", peak, budget);
    std::vector<apm_task> tasks((size_t)n_tasks);
    if (n_tasks > 1) {  // one entry short
        int64_t cap = n_tasks - 1;
        if (apm_schedule_plan(off.data(), pages.data(), bytes.data(), L, with_last ? last.data() : nullptr, P,
                              page_bytes, budget, tasks.data(), &cap, nullptr) != APM_ERANGE) die("short task buffer accepted");
    }
    int64_t cap = n_tasks;
    if (apm_schedule_plan(off.data(), pages.data(), bytes.data(), L, with_last ? last.data() : nullptr, P,
                          page_bytes, budget, tasks.data(), &cap, &peak) != APM_OK) die("plan fill");
    std::vector<char> moved((size_t)P, 0);
    int64_t computes = 0;
    for (const apm_task& t : tasks) {
        if (t.op == APM_TASK_MOVE_TO_GPU) {
            if (t.target < 0 || t.target >= P || moved[(size_t)t.target]) die("movement target", t.target);
            if (t.trigger_id < 0 || t.trigger_id > owner[(size_t)t.target]) die("movement after its layer", t.target, t.trigger_id);
            if (t.trigger_id > computes) die("trigger ahead of the schedule", t.trigger_id, computes);
            moved[(size_t)t.target] = 1;
        } else if (t.op == APM_TASK_COMPUTE) {
            if (t.target != computes || t.trigger_id != computes) die("compute order", t.target, computes);
            for (int64_t k = off[(size_t)computes]; k < off[(size_t)computes + 1]; ++k)
                if (!moved[(size_t)pages[(size_t)k]]) die("layer computed before its page arrived", computes, pages[(size_t)k]);
            ++computes;
        } else {
            die("unknown task op", t.op);
        }
    }
    if (computes != L) die("compute count", computes, L);
}

void plan_errors() {
    int64_t n_tasks = 0;
    int64_t off[2] = {0, 1}, pages[1] = {0}, bytes[1] = {0};
    if (apm_schedule_plan(off, pages, bytes, 1, nullptr, 1, 16, 100, nullptr, nullptr, nullptr) != APM_EINVAL) die("NULL n_tasks accepted");
    if (apm_schedule_plan(off, pages, bytes, 1, nullptr, 1, 0, 100, nullptr, &n_tasks, nullptr) != APM_EINVAL) die("page_bytes 0 accepted");
    if (apm_schedule_plan(off, pages, bytes, 1, nullptr, 2, 16, 100, nullptr, &n_tasks, nullptr) != APM_EINVAL) die("page count mismatch accepted");
    if (apm_schedule_plan(off, pages, bytes, 1, nullptr, 1, INT64_MAX / 2, 100, nullptr, &n_tasks, nullptr) != APM_ENOMEM) die("huge page fits?");
    if (apm_schedule_plan(nullptr, nullptr, nullptr, 0, nullptr, 0, 16, 0, nullptr, &n_tasks, nullptr) != APM_OK || n_tasks != 0) die("empty trace");
    {  // offsets that run past the page list must be refused before the list is read through them
        std::vector<int64_t> off3 = {0, 5, 1}, pages3 = {0}, bytes3 = {0, 0};
        if (apm_schedule_plan(off3.data(), pages3.data(), bytes3.data(), 2, nullptr, 1, 16, 100, nullptr, &n_tasks, nullptr) != APM_EINVAL) die("offsets beyond the list accepted");
    }
    int64_t off2[3] = {0, 2, 1};
    int64_t pages2[2] = {0, 1}, bytes2[2] = {0, 0};
    if (apm_schedule_plan(off2, pages2, bytes2, 2, nullptr, 1, 16, 100, nullptr, &n_tasks, nullptr) == APM_OK) die("decreasing offsets accepted");
}

}  // namespace

int main(int argc, char** argv) {
    const int cases = argc > 1 ? std::atoi(argv[1]) : 2000;
    Rng r{0x2303028680ull};
    pack_errors();
    plan_errors();
    for (int i = 0; i < cases; ++i) pack_case(r);
    for (int i = 0; i < cases; ++i) plan_case(r);
    std::printf("ok %d\n", cases);
    return 0;
}
