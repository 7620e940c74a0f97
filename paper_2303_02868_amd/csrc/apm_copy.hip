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
// is the bound, not the GPU, and one kernel driving both directions keeps them balanced where two
// independent copies (DMA or kernels) compete (measured: 49 GB/s each way against 44-48, and
// against 28 when the runtime happens to serialise its two copy queues).
constexpr int kDuplexItem = 4096;  // bytes per class, direction and wavefront iteration
constexpr int kDuplexU = kDuplexItem / (64 * 16);

template <bool FULL>
__device__ __forceinline__ void duplex_item(const DuplexCopy& a, int64_t base) {
    typedef const u32x4 __attribute__((address_space(1))) * In;
    typedef u32x4 __attribute__((address_space(1))) * Out;
    u32x4 vin[3][kDuplexU], vout[3][kDuplexU];
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u) {
            const int64_t off = base + (int64_t)u * 1024;
            if (FULL || off < a.in_bytes) vin[k][u] = __builtin_nontemporal_load((In)(a.in_src[k] + off));
            if (FULL || off < a.out_bytes) vout[k][u] = __builtin_nontemporal_load((In)(a.out_src[k] + off));
        }
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int u = 0; u < kDuplexU; ++u) {
            const int64_t off = base + (int64_t)u * 1024;
            if (FULL || off < a.in_bytes) __builtin_nontemporal_store(vin[k][u], (Out)(a.in_dst[k] + off));
            if (FULL || off < a.out_bytes) __builtin_nontemporal_store(vout[k][u], (Out)(a.out_dst[k] + off));
        }
}

__global__ __launch_bounds__(1024) void apm_duplex_copy_kernel(DuplexCopy a, int n_workers) {
    const int lane = (int)threadIdx.x & 63;
    const int waves_per_wg = (int)blockDim.x / 64;
    const int worker = (int)blockIdx.x * waves_per_wg + __builtin_amdgcn_readfirstlane((int)threadIdx.x / 64);
    if (worker >= n_workers) return;
    const int64_t longer = a.in_bytes > a.out_bytes ? a.in_bytes : a.out_bytes;
    const int64_t n_items = (longer + kDuplexItem - 1) / kDuplexItem;
#pragma unroll 1
    for (int64_t item = worker; item < n_items; item += n_workers) {
        const int64_t base = item * kDuplexItem + (int64_t)lane * 16;
        const int64_t end = (item + 1) * kDuplexItem;
        if (end <= a.in_bytes && end <= a.out_bytes) duplex_item<true>(a, base);
        else duplex_item<false>(a, base);  // byte counts are multiples of 16: a vector is in or out
    }
}

}  // namespace

hipError_t launch_duplex_copy(const DuplexCopy& d, int wavefronts, int per_wg, hipStream_t s) {
    const int64_t longer = d.in_bytes > d.out_bytes ? d.in_bytes : d.out_bytes;
    if (longer <= 0) return hipSuccess;
    const int64_t n_items = (longer + kDuplexItem - 1) / kDuplexItem;
    const int workers = (int)(n_items < wavefronts ? n_items : wavefronts);
    if (per_wg < 1 || per_wg > 16) per_wg = 1;
    hipLaunchKernelGGL(apm_duplex_copy_kernel, dim3((unsigned)((workers + per_wg - 1) / per_wg)),
                       dim3((unsigned)(per_wg * 64)), 0, s, d, workers);
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
