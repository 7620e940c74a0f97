// Gather / scatter between contiguous tensors and page storage: a list of (src, dst, nbytes)
// segments, each inside one page, copied bit for bit.  HBM-bound (read n + write n bytes).
//
// grid.y walks the segments, grid.x the fixed-size chunks of a segment; chunks beyond a segment's end
// exit at once.  Segments whose source and destination are both 16-byte aligned move 128 bits per
// lane with contiguous wavefront accesses; any other alignment falls back to the widest unit that
// divides both addresses and the length.
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

// Bytes of item `item` of a batch that lie inside its page's used extent (<= 0: none).  With a
// page table, a page is a whole number of items (items_per_page), so an item lies in one page.
__device__ __forceinline__ int duplex_limit(const DuplexCopy& a, unsigned item, unsigned batch_items,
                                            int64_t batch_bytes, int64_t first_page) {
    if (item >= batch_items) return 0;
    if (!a.used) {
        const int64_t left = batch_bytes - (int64_t)item * kDuplexItem;
        return left < kDuplexItem ? (int)left : kDuplexItem;
    }
    const unsigned page = item / a.items_per_page;
    const int64_t in_page = (int64_t)(item - page * a.items_per_page) * kDuplexItem;
    const int64_t used_bytes = (((int64_t)a.used[first_page + page] + 7) & ~(int64_t)7) * 4;
    const int64_t left = used_bytes - in_page;  // pages go up to 2^30 elements: 64-bit
    return left < kDuplexItem ? (int)(left < 0 ? 0 : left) : kDuplexItem;
}

template <bool FULL>
__device__ __forceinline__ void duplex_item(const DuplexCopy& a, int64_t base, int lane_off, int lim_in, int lim_out) {
    typedef const u32x4 __attribute__((address_space(1))) * In;
    typedef u32x4 __attribute__((address_space(1))) * Out;
    u32x4 vin[3][kDuplexU], vout[3][kDuplexU];
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u)
            if (FULL || lane_off + u * 1024 < lim_in) vin[k][u] = __builtin_nontemporal_load((In)(a.in_src[k] + base + u * 1024));
    __builtin_amdgcn_sched_barrier(0);  // keep the order written here: host reads first
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u)
            if (FULL || lane_off + u * 1024 < lim_out) vout[k][u] = __builtin_nontemporal_load((In)(a.out_src[k] + base + u * 1024));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u)
            if (FULL || lane_off + u * 1024 < lim_out) __builtin_nontemporal_store(vout[k][u], (Out)(a.out_dst[k] + base + u * 1024));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u)
            if (FULL || lane_off + u * 1024 < lim_in) __builtin_nontemporal_store(vin[k][u], (Out)(a.in_dst[k] + base + u * 1024));
}

__global__ __launch_bounds__(1024) void apm_duplex_copy_kernel(DuplexCopy a, int n_workers) {
    const int lane = (int)threadIdx.x & 63;
    const int waves_per_wg = (int)blockDim.x / 64;
    const int worker = (int)blockIdx.x * waves_per_wg + __builtin_amdgcn_readfirstlane((int)threadIdx.x / 64);
    if (worker >= n_workers) return;
    const unsigned in_items = (unsigned)((a.in_bytes + kDuplexItem - 1) / kDuplexItem);
    const unsigned out_items = (unsigned)((a.out_bytes + kDuplexItem - 1) / kDuplexItem);
    const unsigned n_items = in_items > out_items ? in_items : out_items;
    const int lane_off = lane * 16;
    // The used extents of the next item are looked up (two dependent scalar loads) while the
    // current item's data is in flight, so the lookup never delays the issue of the data loads.
    unsigned item = (unsigned)worker;
    int lim_in = duplex_limit(a, item, in_items, a.in_bytes, a.in_first_page);
    int lim_out = duplex_limit(a, item, out_items, a.out_bytes, a.out_first_page);
#pragma unroll 1
    while (item < n_items) {
        const unsigned next = item + (unsigned)n_workers;
        const int64_t base = (int64_t)item * kDuplexItem + lane_off;
        const int cur_in = lim_in, cur_out = lim_out;
        lim_in = duplex_limit(a, next, in_items, a.in_bytes, a.in_first_page);
        lim_out = duplex_limit(a, next, out_items, a.out_bytes, a.out_first_page);
        // byte counts and used extents are multiples of 16: a 16-byte vector is wholly in or out
        if (cur_in >= kDuplexItem && cur_out >= kDuplexItem) duplex_item<true>(a, base, lane_off, cur_in, cur_out);
        else if (cur_in > 0 || cur_out > 0) duplex_item<false>(a, base, lane_off, cur_in, cur_out);
        item = next;
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
    hipLaunchKernelGGL(apm_duplex_copy_kernel, dim3((unsigned)((workers + per_wg - 1) / per_wg)),
                       dim3((unsigned)(per_wg * 64)), 0, s, a, workers);
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
