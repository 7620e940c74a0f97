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

}  // namespace

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
