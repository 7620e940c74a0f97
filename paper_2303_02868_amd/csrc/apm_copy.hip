// Gather / scatter between contiguous tensors and page storage: a list of (src, dst, nbytes)
// segments, each inside one page, copied bit for bit.  HBM-bound (read n + write n bytes).
//
// grid.y walks the segments, grid.x the fixed-size chunks of a segment; chunks beyond a segment's end
// exit at once.  Segments whose source and destination are both 16-byte aligned move 128 bits per
// lane with contiguous wavefront accesses; any other alignment falls back to the widest unit that
// divides both addresses and the length.
#include <cstdlib>
#include "apm_internal.h"

namespace apm {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#ifndef APM_COPY_THREADS
#define APM_COPY_THREADS 256
#endif
#ifndef APM_COPY_U
#define APM_COPY_U 1   // 128-bit vectors per lane; one per lane measured fastest for a plain copy
#endif
constexpr int kThreads = APM_COPY_THREADS;
constexpr int kVecPerLane = APM_COPY_U;
constexpr int64_t kChunk = (int64_t)kThreads * 16 * kVecPerLane;
constexpr int kMaxGridY = 65535;

// Fallback for segments whose addresses are not both 16-byte aligned: the widest unit that
// divides both addresses and the length.  Kept out of line and not unrolled so that it does not
// inflate the register footprint of the aligned path.
template <typename T>
__device__ __noinline__ void copy_units(const char* src, char* dst, int64_t n_units) {
    const T* s = reinterpret_cast<const T*>(src);
    T* d = reinterpret_cast<T*>(dst);
#pragma unroll 1
    for (int64_t k = threadIdx.x; k < n_units; k += kThreads) d[k] = s[k];
}

__global__ __launch_bounds__(kThreads) void apm_seg_copy_kernel(const SegDesc* descs, int64_t seg_offset) {
    const SegDesc d = descs[seg_offset + blockIdx.y];
    const int64_t start = (int64_t)blockIdx.x * kChunk;
    if (start >= d.nbytes) return;
    const int64_t len = d.nbytes - start < kChunk ? d.nbytes - start : kChunk;
    const char* src = static_cast<const char*>(d.src) + start;
    char* dst = static_cast<char*>(d.dst) + start;
    const uintptr_t mis = reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst);
    if ((mis & 15u) == 0) {
        const int nvec = (int)(len >> 4);
        const u32x4* s = reinterpret_cast<const u32x4*>(src);
        u32x4* o = reinterpret_cast<u32x4*>(dst);
        u32x4 r[kVecPerLane];
#pragma unroll
        for (int k = 0; k < kVecPerLane; ++k) {
            const int vi = k * kThreads + (int)threadIdx.x;
            if (vi < nvec) r[k] = __builtin_nontemporal_load(s + vi);
        }
#pragma unroll
        for (int k = 0; k < kVecPerLane; ++k) {
            const int vi = k * kThreads + (int)threadIdx.x;
            if (vi < nvec) __builtin_nontemporal_store(r[k], o + vi);
        }
        const int tail = (int)(len & 15);  // only the last chunk of a segment can have one
        if ((int)threadIdx.x < tail) dst[((int64_t)nvec << 4) + threadIdx.x] = src[((int64_t)nvec << 4) + threadIdx.x];
    } else if (((mis | (uintptr_t)len) & 7u) == 0) {
        copy_units<uint64_t>(src, dst, len >> 3);
    } else if (((mis | (uintptr_t)len) & 3u) == 0) {
        copy_units<uint32_t>(src, dst, len >> 2);
    } else if (((mis | (uintptr_t)len) & 1u) == 0) {
        copy_units<uint16_t>(src, dst, len >> 1);
    } else {
        copy_units<uint8_t>(src, dst, len);
    }
}

// Both directions of a staged batch exchange in one kernel: the fp32 classes of an incoming batch
// move from pinned host pages into a staging slot while those of an outgoing batch move from
// another slot back to their host pages.  A fixed, small number of wavefronts strides over 4 KiB
// items (one 1 KiB span per wavefront instruction, 4 per class and direction in flight); the link
// is the bound, not the GPU.  One kernel driving both directions keeps them balanced: measured on
// 3 x 1 GiB each way, 49.3 GB/s each way with 48 wavefronts, against 40-42 when half of the
// wavefronts serve each direction (or two kernels do), 48.6 for two runtime copies when the
// runtime overlaps them, and 28 when it does not.  Within an item all host reads are issued first
// (they have the longest latency), then the staging reads; the host writes go out before the
// staging writes (interleaving the two directions instruction by instruction: 47.2 GB/s).
// Only the used extent of each page is moved: the update never touches the rest.
constexpr int kDuplexItem = 4096;  // bytes per class, direction and wavefront iteration
constexpr int kDuplexU = kDuplexItem / (64 * 16);

// A wavefront's position in one direction's run of pages.  A wavefront visits the items congruent
// to its number modulo the wavefront count, and of those only the ones that hold used bytes: items
// beyond a page's used extent are not visited one by one, the cursor hops along its stride to the
// next page.  Skipping them (instead of spending an iteration on an item that is empty in one
// direction) keeps the two directions of an exchange in step when their nearly empty pages sit at
// different positions -- a fifth of the items of a 32-page exchange on a GPT-shaped layout.
// With a page table a page is a whole number of items (items_per_page), so an item lies in one
// page; without one the run is treated as a single page.
struct DuplexCursor {
    unsigned item;        // index in the run (>= n_items: nothing left)
    unsigned page;        // page of the run the item lies in
    unsigned in_page;     // index of the item within that page
    unsigned page_items;  // items of that page that hold used bytes
    int tail;             // bytes of the last of them
    int limit;            // bytes of the current item to move (0: nothing left)
};

struct DuplexRun {
    const int32_t* used;  // page table entry of the run's first page, or nullptr
    unsigned n_items, items_per_page, stride;
    int64_t bytes;
};

__device__ __forceinline__ void duplex_page(const DuplexRun& r, DuplexCursor& c) {
    // The page table does not change while the kernel runs; read through the constant address
    // space it is a scalar load that only its own use waits for (as a plain global load it is a
    // vector load followed by a wait for every outstanding memory operation).
    typedef const int32_t __attribute__((address_space(4))) * ConstTable;
    const int64_t used_bytes = (((int64_t)((ConstTable)r.used)[c.page] + 7) & ~(int64_t)7) * 4;  // up to 2^32
    c.page_items = (unsigned)((used_bytes + kDuplexItem - 1) / kDuplexItem);
    c.tail = (int)(used_bytes - (int64_t)(c.page_items ? c.page_items - 1 : 0) * kDuplexItem);
}

// Settles the cursor on the first item at or after its position, on its stride, that holds used
// bytes.  Every turn of the loop either returns or moves on to a later page of the run.
__device__ __forceinline__ void duplex_settle(const DuplexRun& r, DuplexCursor& c) {
#pragma unroll 1
    for (;;) {
        if (c.item >= r.n_items) {
            c.limit = 0;
            return;
        }
        if (c.in_page >= r.items_per_page) {  // crossed into the next page (item < n_items: it exists)
            c.in_page -= r.items_per_page;
            ++c.page;
            duplex_page(r, c);
            continue;
        }
        if (c.in_page < c.page_items) {
            c.limit = c.in_page + 1 == c.page_items ? c.tail : kDuplexItem;
            return;
        }
        const unsigned hops = (r.items_per_page - c.in_page + r.stride - 1) / r.stride;  // >= 1
        c.item += hops * r.stride;
        c.in_page += hops * r.stride;
    }
}

__device__ __forceinline__ void duplex_start(const DuplexRun& r, DuplexCursor& c, unsigned worker) {
    c.item = c.in_page = worker;
    c.page = 0;
    c.limit = 0;
    if (r.used) {
        c.page_items = 0;
        c.tail = 0;
        if (r.n_items > 0) duplex_page(r, c);
    } else {
        c.page_items = r.n_items;
        c.tail = (int)(r.bytes - (int64_t)(r.n_items ? r.n_items - 1 : 0) * kDuplexItem);
    }
    duplex_settle(r, c);
}

typedef const u32x4 __attribute__((address_space(1))) * DuplexIn;
typedef u32x4 __attribute__((address_space(1))) * DuplexOut;

// One item of each direction: all loads, then all stores, in one basic block (FULL) so that the
// stores wait for their own loads only, in issue order.
template <bool FULL, bool WT>
__device__ __forceinline__ void duplex_item(const DuplexCopy& a, int64_t base_in, int64_t base_out, int lane_off,
                                            int lim_in, int lim_out) {
    u32x4 vin[3][kDuplexU], vout[3][kDuplexU];
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u)
            if (FULL || lane_off + u * 1024 < lim_in) vin[k][u] = __builtin_nontemporal_load((DuplexIn)(a.in_src[k] + base_in + u * 1024));
    __builtin_amdgcn_sched_barrier(0);  // keep the order written here: host reads first
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u)
            if (FULL || lane_off + u * 1024 < lim_out) vout[k][u] = __builtin_nontemporal_load((DuplexIn)(a.out_src[k] + base_out + u * 1024));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u)
            if (FULL || lane_off + u * 1024 < lim_out) {
                // WT: written through at system scope.  A non-temporal store to host memory may rest
                // in the L2 as a dirty line, and the write-back that ends every kernel of any other
                // stream then pushes it across PCIe: those kernels pay for this kernel's writes.
                DuplexOut q = (DuplexOut)(a.out_dst[k] + base_out + u * 1024);
                // (hand-written because no builtin takes a cache policy for a 128-bit global store.
                // The compiler does not know that this is a store whose data registers are read a
                // little after issue -- for its own stores of more than 64 bits it keeps the next
                // instruction from overwriting them -- so the wait states go in by hand.)
                if (WT) asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(q), "v"(vout[k][u]) : "memory");
                else __builtin_nontemporal_store(vout[k][u], q);
            }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u)
            if (FULL || lane_off + u * 1024 < lim_in) __builtin_nontemporal_store(vin[k][u], (DuplexOut)(a.in_dst[k] + base_in + u * 1024));
}

template <bool WT>
__global__ __launch_bounds__(1024) void apm_duplex_copy_kernel(DuplexCopy a, int n_workers) {
    const int lane = (int)threadIdx.x & 63;
    const int waves_per_wg = (int)blockDim.x / 64;
    const int worker = (int)blockIdx.x * waves_per_wg + __builtin_amdgcn_readfirstlane((int)threadIdx.x / 64);
    if (worker >= n_workers) return;
    const unsigned in_items = (unsigned)((a.in_bytes + kDuplexItem - 1) / kDuplexItem);
    const unsigned out_items = (unsigned)((a.out_bytes + kDuplexItem - 1) / kDuplexItem);
    const int lane_off = lane * 16;
    // Each direction has its own cursor over the items that hold used bytes; the next positions
    // are worked out (scalar arithmetic, a scalar load per page) before the current item's data moves.
    const unsigned ipp = a.used ? a.items_per_page : 0xffffffffu;
    const DuplexRun rin{a.used ? a.used + a.in_first_page : nullptr, in_items, ipp, (unsigned)n_workers, a.in_bytes};
    const DuplexRun rout{a.used ? a.used + a.out_first_page : nullptr, out_items, ipp, (unsigned)n_workers, a.out_bytes};
    DuplexCursor in, out;
    duplex_start(rin, in, (unsigned)worker);
    duplex_start(rout, out, (unsigned)worker);
#pragma unroll 1
    while (in.limit > 0 || out.limit > 0) {
        // byte counts and used extents are multiples of 16: a 16-byte vector is wholly in or out
        const int cur_in = in.limit, cur_out = out.limit;
        const int64_t base_in = (int64_t)in.item * kDuplexItem + lane_off;
        const int64_t base_out = (int64_t)out.item * kDuplexItem + lane_off;
        if (cur_in > 0) {
            in.item += (unsigned)n_workers;
            in.in_page += (unsigned)n_workers;
            duplex_settle(rin, in);
        }
        if (cur_out > 0) {
            out.item += (unsigned)n_workers;
            out.in_page += (unsigned)n_workers;
            duplex_settle(rout, out);
        }
        if (cur_in >= kDuplexItem && cur_out >= kDuplexItem) duplex_item<true, WT>(a, base_in, base_out, lane_off, cur_in, cur_out);
        else duplex_item<false, WT>(a, base_in, base_out, lane_off, cur_in, cur_out);
    }
}

}  // namespace

hipError_t launch_duplex_copy(const DuplexCopy& d, int wavefronts, int per_wg, hipStream_t s) {
    const int64_t longer = d.in_bytes > d.out_bytes ? d.in_bytes : d.out_bytes;
    if (longer <= 0) return hipSuccess;
    const int64_t n_items = (longer + kDuplexItem - 1) / kDuplexItem;
    const int workers = (int)(n_items < wavefronts ? n_items : wavefronts);
    if (per_wg < 1 || per_wg > 16) per_wg = 1;
    DuplexCopy a = d;
    if (a.page_bytes <= 0 || a.page_bytes % kDuplexItem != 0) a.used = nullptr;
    a.items_per_page = a.used ? (uint32_t)(a.page_bytes / kDuplexItem) : 0u;
    if (n_items >= ((int64_t)1 << 31)) return hipErrorInvalidValue;  // 8 TiB per class and kernel
    const dim3 grid((unsigned)((workers + per_wg - 1) / per_wg)), block((unsigned)(per_wg * 64));
    if (a.host_store_policy != 0) hipLaunchKernelGGL(apm_duplex_copy_kernel<true>, grid, block, 0, s, a, workers);
    else hipLaunchKernelGGL(apm_duplex_copy_kernel<false>, grid, block, 0, s, a, workers);
    return hipGetLastError();
}

hipError_t launch_seg_copy(const SegDesc* d_descs, int64_t n, int64_t max_bytes, hipStream_t s) {
    if (n == 0 || max_bytes == 0) return hipSuccess;
    const unsigned nx = (unsigned)((max_bytes + kChunk - 1) / kChunk);
    for (int64_t off = 0; off < n; off += kMaxGridY) {
        const int64_t ny = n - off < kMaxGridY ? n - off : kMaxGridY;
        hipLaunchKernelGGL(apm_seg_copy_kernel, dim3(nx, (unsigned)ny), dim3(kThreads), 0, s, d_descs, off);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace apm
