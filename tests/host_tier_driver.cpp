// Drives the file tier's host-side thread choreography (apm_io.h: I/O thread pool + window chain)
// on the CPU, with a plain loop standing in for the update kernel.  Built with ThreadSanitizer (and
// once more with ASan + UBSan) by tests/test_host_sanitizers.py.
//
// usage: host_tier_driver DIR
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "apm_io.h"

using apm::io::IoPool;
using apm::io::WindowChain;

namespace {

[[noreturn]] void die(const char* what, long long a = 0, long long b = 0) {
    std::fprintf(stderr, "tier driver check failed: %s (%lld, %lld)\n", what, a, b);
    std::exit(1);
}

struct Files {
    int fd[3] = {-1, -1, -1};
    std::string path[3];
    ~Files() {
        for (int c = 0; c < 3; ++c) {
            if (fd[c] >= 0) close(fd[c]);
            if (!path[c].empty()) unlink(path[c].c_str());
        }
    }
};

// Element e of page p in class c starts as this.
float initial(int c, int64_t p, int64_t e) { return (float)(c * 1000000 + p * 1000 + e % 997); }

// false: the file system does not take the open flags (unbuffered I/O on a memory file system).
bool make_files(Files& f, const std::string& dir, const char* tag, int64_t n_pages, int64_t page_floats, int oflags) {
    for (int c = 0; c < 3; ++c) {
        f.path[c] = dir + "/tier_" + tag + "_" + std::to_string(c) + ".bin";
        f.fd[c] = open(f.path[c].c_str(), O_RDWR | O_CREAT | O_TRUNC | oflags, 0600);
        if (f.fd[c] < 0 && errno == EINVAL && oflags != 0) return false;
        if (f.fd[c] < 0) die("open", c, errno);
        std::vector<float> page((size_t)page_floats);
        for (int64_t p = 0; p < n_pages; ++p) {
            for (int64_t e = 0; e < page_floats; ++e) page[(size_t)e] = initial(c, p, e);
            if (apm::io::io_piece(f.fd[c], reinterpret_cast<char*>(page.data()), page.size() * sizeof(float),
                                  (off_t)((size_t)p * page.size() * sizeof(float)), true, oflags != 0) != 0)
                die("initial write", c, p);
        }
    }
    return true;
}

// n_steps passes, each adding (1 + class) to every element; then the files are read back.
void case_roundtrip(const std::string& dir, const char* tag, int64_t n_pages, int64_t page_floats, int64_t B,
                    int n_slots, int threads, bool direct, int n_steps) {
    Files f;
    if (!make_files(f, dir, tag, n_pages, page_floats, direct ? O_DIRECT : 0)) {
        std::printf("case %s skipped: no unbuffered I/O in %s\n", tag, dir.c_str());
        return;
    }
    const size_t pb = (size_t)page_floats * sizeof(float);
    std::vector<std::vector<char>> win(3, std::vector<char>((size_t)n_slots * (size_t)B * pb));
    char* w[3] = {win[0].data(), win[1].data(), win[2].data()};
    {
        IoPool pool(threads);
        WindowChain chain(&pool, f.fd, w, pb, B, n_slots, direct);
        int64_t seen_pages = 0;
        for (int s = 0; s < n_steps; ++s) {
            seen_pages = 0;
            const int rc = chain.run(n_pages, [&](int64_t b, int slot, int64_t first, int64_t nb) {
                if (first != b * B || slot != (int)(b % n_slots)) die("batch geometry", b, first);
                for (int c = 0; c < 3; ++c) {
                    float* x = reinterpret_cast<float*>(chain.slot_base(c, slot));
                    for (int64_t e = 0; e < nb * page_floats; ++e) x[e] += (float)(1 + c);
                }
                seen_pages += nb;
                return true;
            });
            if (rc != 0) die("run failed", rc, s);
            if (seen_pages != n_pages) die("pages processed", seen_pages, n_pages);
        }
    }
    std::vector<float> page((size_t)page_floats);
    for (int c = 0; c < 3; ++c)
        for (int64_t p = 0; p < n_pages; ++p) {
            if (apm::io::io_piece(f.fd[c], reinterpret_cast<char*>(page.data()), pb, (off_t)((size_t)p * pb), false, direct) != 0)
                die("read back", c, p);
            for (int64_t e = 0; e < page_floats; ++e)
                if (page[(size_t)e] != initial(c, p, e) + (float)(n_steps * (1 + c))) die("value after the steps", c, p * page_floats + e);
        }
}

// Only some pages pass through the window (the pages of a step that received a gradient): the
// listed pages change, the others keep their bits, and only the listed ones are read and written.
void case_list(const std::string& dir) {
    const int64_t n_pages = 50, page_floats = 2048, B = 4;
    const int n_slots = 3;
    Files f;
    make_files(f, dir, "list", n_pages, page_floats, 0);
    const size_t pb = (size_t)page_floats * sizeof(float);
    std::vector<std::vector<char>> win(3, std::vector<char>((size_t)n_slots * (size_t)B * pb));
    char* w[3] = {win[0].data(), win[1].data(), win[2].data()};
    const std::vector<int64_t> pages = {0, 1, 2, 7, 9, 10, 11, 12, 13, 20, 33, 34, 48, 49};  // runs and singles
    IoPool pool(4);
    WindowChain chain(&pool, f.fd, w, pb, B, n_slots, false);
    int64_t seen = 0;
    const int rc = chain.run_list(pages.data(), (int64_t)pages.size(), [&](int64_t b, int slot, int64_t first, int64_t nb) {
        if (first != b * B) die("list batch geometry", b, first);
        for (int c = 0; c < 3; ++c) {
            float* x = reinterpret_cast<float*>(chain.slot_base(c, slot));
            for (int64_t j = 0; j < nb; ++j) {
                const int64_t p = pages[(size_t)(first + j)];
                for (int64_t e = 0; e < page_floats; ++e) {
                    if (x[j * page_floats + e] != initial(c, p, e)) die("window holds the wrong page", p, e);
                    x[j * page_floats + e] = -(float)(p + 1);
                }
            }
        }
        seen += nb;
        return true;
    });
    if (rc != 0 || seen != (int64_t)pages.size()) die("list run", rc, seen);
    int64_t rd = 0, wr = 0;
    chain.io_bytes(&rd, &wr);
    if (rd != 3 * (int64_t)pages.size() * (int64_t)pb || wr != rd) die("bytes moved for a list", rd, wr);
    std::vector<float> page((size_t)page_floats);
    for (int c = 0; c < 3; ++c)
        for (int64_t p = 0; p < n_pages; ++p) {
            if (apm::io::io_full(f.fd[c], reinterpret_cast<char*>(page.data()), pb, (off_t)((size_t)p * pb), false) != 0) die("read back");
            bool listed = false;
            for (int64_t q : pages) listed = listed || q == p;
            for (int64_t e = 0; e < page_floats; ++e)
                if (page[(size_t)e] != (listed ? -(float)(p + 1) : initial(c, p, e))) die("page after a list run", p, e);
        }
    if (chain.run_list(pages.data(), 0, [&](int64_t, int, int64_t, int64_t) { return true; }) != 0) die("empty list");
}

// A file that is shorter than the pool: reads beyond its end fail; the run must report the error,
// process nothing after it, and return with nothing in flight.
void case_short_file(const std::string& dir) {
    const int64_t n_pages = 23, page_floats = 1024, B = 3;
    const int n_slots = 2;
    Files f;
    make_files(f, dir, "short", n_pages, page_floats, 0);
    const size_t pb = (size_t)page_floats * sizeof(float);
    if (ftruncate(f.fd[1], (off_t)(10 * pb)) != 0) die("ftruncate");
    std::vector<std::vector<char>> win(3, std::vector<char>((size_t)n_slots * (size_t)B * pb));
    char* w[3] = {win[0].data(), win[1].data(), win[2].data()};
    IoPool pool(4);
    WindowChain chain(&pool, f.fd, w, pb, B, n_slots, false);
    int64_t processed = 0;
    const int rc = chain.run(n_pages, [&](int64_t, int, int64_t, int64_t nb) { processed += nb; return true; });
    if (rc != EIO) die("short file not reported", rc);
    if (processed > 12) die("batches processed after the failed read", processed);
    // the chain is reusable: a run over the part that exists succeeds
    if (chain.run(9, [&](int64_t, int, int64_t, int64_t) { return true; }) != 0) die("run after a failure");
}

// The processing side gives up (a failed kernel launch): nothing more is written, the run drains.
void case_refusal(const std::string& dir) {
    const int64_t n_pages = 40, page_floats = 512, B = 4;
    const int n_slots = 3;
    Files f;
    make_files(f, dir, "refuse", n_pages, page_floats, 0);
    const size_t pb = (size_t)page_floats * sizeof(float);
    std::vector<std::vector<char>> win(3, std::vector<char>((size_t)n_slots * (size_t)B * pb));
    char* w[3] = {win[0].data(), win[1].data(), win[2].data()};
    IoPool pool(3);
    WindowChain chain(&pool, f.fd, w, pb, B, n_slots, false);
    int64_t calls = 0;
    const int rc = chain.run(n_pages, [&](int64_t b, int slot, int64_t, int64_t nb) {
        ++calls;
        float* x = reinterpret_cast<float*>(chain.slot_base(0, slot));
        for (int64_t e = 0; e < nb * page_floats; ++e) x[e] = -1.0f;
        return b < 4;  // batch 4 is refused
    });
    if (rc != -1) die("refusal not reported", rc);
    if (calls != 5) die("process called after its refusal", calls);
    std::vector<float> page((size_t)page_floats);
    for (int64_t p = 0; p < n_pages; ++p) {
        if (apm::io::io_full(f.fd[0], reinterpret_cast<char*>(page.data()), pb, (off_t)((size_t)p * pb), false) != 0) die("read back");
        const bool written = p < 4 * B;
        for (int64_t e = 0; e < page_floats; ++e)
            if (page[(size_t)e] != (written ? -1.0f : initial(0, p, e))) die("page state after a refusal", p, e);
    }
}

}  // namespace

int main(int argc, char** argv) {
    if (argc < 2) die("usage: host_tier_driver DIR");
    const std::string dir = argv[1];
    case_roundtrip(dir, "a", 37, 1024, 5, 2, 3, false, 3);       // ragged last batch
    case_roundtrip(dir, "b", 16, 4096, 16, 3, 8, false, 2);      // one batch, more slots than batches
    case_roundtrip(dir, "c", 64, 256, 1, 4, 2, false, 2);        // one page per batch
    case_roundtrip(dir, "d", 5, 3 << 20, 2, 2, 4, false, 1);     // batches of several I/O pieces
    case_roundtrip(dir, "e", 24, 2048, 4, 2, 4, true, 2);        // unbuffered, through the bounce buffers
    case_list(dir);
    case_short_file(dir);
    case_refusal(dir);
    std::printf("ok\n");
    return 0;
}
