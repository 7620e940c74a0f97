// Page AdamW kernels for gfx950:
//   apm_grad_reduce_kernel    per (page, slice) sum of squares (fp64) and any-nonzero of g16
//   apm_grad_finalize_kernel  per page: norm, clip scale, skip decision -> the page's record
//   apm_page_meta_kernel      the page records when no reduce pass is needed
//   apm_adamw_kernel          the fused update (optionally gathering g16 from / scattering p16 to
//                             the caller's tensors), one workgroup per page slice
//   apm_adamw_stride_kernel   the same slice body run by a fixed, small number of wavefronts that
//                             stride over all slices (fp32 classes in host memory across PCIe)
//   apm_grad_accum_kernel     g' += g for the buffered gradient of the delayed path
//
// All are HBM-bandwidth bound (no reuse, ~50 VALU operations per element at most), so the design
// is about memory access only: every wavefront instruction touches one fully contiguous span
// (1 KiB for the 128-bit fp32 accesses, 512 B for the 64-bit bf16 accesses), each lane keeps
// several independent loads in flight, and a workgroup never straddles a page.
//
// Work decomposition: grid.y walks the listed pages, grid.x the fixed-size slices of a page;
// slices that start beyond the page's used extent exit at once.  The page table (`used`) is read
// on the device; the host, which knows the extents from the layout, only sizes the grids (pages
// grouped into extent classes) so that few workgroups are launched for nothing.
#include "apm_internal.h"

namespace apm {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kWave = 64;

__device__ __forceinline__ double shfl_xor_f64(double x, int off) {
    int lo = __double2loint(x), hi = __double2hiint(x);
    lo = __shfl_xor(lo, off, kWave);
    hi = __shfl_xor(hi, off, kWave);
    return __hiloint2double(hi, lo);
}

// Sum over the wavefront in a fixed butterfly order; every lane ends with the same value.
__device__ __forceinline__ double wave_sum_f64(double x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += shfl_xor_f64(x, off);
    return x;
}

__device__ __forceinline__ uint32_t wave_or_u32(uint32_t x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x |= (uint32_t)__shfl_xor((int)x, off, kWave);
    return x;
}

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Round-to-nearest-even of an fp32 value to bf16 bits, on the integer representation.
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
    const uint32_t u = __float_as_uint(x);
    // both forms are computed and one is selected: a branch here would split the update kernel's
    // body into basic blocks (see slice_body)
    const uint32_t nan = (u >> 16) | 0x0040u;
    const uint32_t rne = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return (u & 0x7FFFFFFFu) > 0x7F800000u ? nan : rne;
}

// ---- tunables (defaults measured on MI355X; see the sweep notes next to each) ----------------
#ifndef APM_FAST_RCP_SQRT
// 1: hardware 1-ulp reciprocal and square root instead of the correctly rounded sequences.
// Measured slower (6.0 vs 6.25 TB/s): the kernel is not ALU-bound, so the exact forms stay.
#define APM_FAST_RCP_SQRT 0
#endif
#ifndef APM_REDUCE_U
#define APM_REDUCE_U 4          // 128-bit loads in flight per lane in the reduce kernel
#endif
#ifndef APM_UPDATE_THREADS
#define APM_UPDATE_THREADS 64   // one wavefront per page slice
#endif
#ifndef APM_UPDATE_U
#define APM_UPDATE_U 4          // 128-bit vectors per lane and fp32 class
#endif
#ifndef APM_UPDATE_SLICES_SKIP
// Page slices one workgroup walks through when pages may be skipped on the device
// (APM_SKIP_UNTOUCHED).  Dense launches use one slice per workgroup, which is fastest when every
// workgroup has work (5.9 TB/s against 5.7 / 5.3 with 2 / 4 slices); when 7 of 8 pages are
// skipped, the workgroups that only find that out and leave dominate, and 4 slices per workgroup
// cut their number (MoE workload: update 3.03 ms -> 2.61 ms).
#define APM_UPDATE_SLICES_SKIP 4
#endif
#ifndef APM_HOIST_LOADS
#define APM_HOIST_LOADS 1
#endif
#ifndef APM_UPDATE_LDS
// Dynamic LDS requested per workgroup for no purpose other than capping residency at
// 160 KiB / 32 KiB = 5 wavefronts per CU: with four read and four write streams per wavefront,
// more resident wavefronts lower the achieved HBM bandwidth.  Measured on the 1.3 B-parameter
// workload with the single-block slice body (16 loads, then 16 stores in flight per wavefront):
// 5.5 TB/s at 16 wavefronts per CU, 5.6 at 13, 5.9 at 10, 5.7-6.1 at 8, 6.1 at 6, 6.3 at 5,
// 6.0-6.3 at 4, 6.1 at 3, 5.1 at 2.  (The earlier body, whose wavefronts waited for each vector's
// stores, peaked at 8.)
#define APM_UPDATE_LDS 32768
#endif

// Gradient elements [e, e+8) of a page, read from its tenant tensors; elements that belong to no
// tenant (alignment gap, padding) read as zero.  e is a multiple of 8, as every tenant offset is,
// so a vector never straddles the start of the second tenant.
__device__ __forceinline__ u32x4 gather_g8(const PageSegs& s, int e) {
    const int k = (s.n[1] > 0 && e >= s.off[1]) ? 1 : 0;
    const int rel = e - s.off[k];
    const int n = s.n[k];
    u32x4 w = u32x4{0u, 0u, 0u, 0u};
    if (rel >= 0 && rel + 8 <= n) {
        w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(s.g[k] + rel));
    } else if (rel >= 0 && rel < n) {  // last, partial vector of the tensor: never read past its end
        const uint16_t* src = s.g[k] + rel;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (rel + j < n) w[j >> 1] |= (uint32_t)src[j] << (16 * (j & 1));
    }
    return w;
}

__device__ __forceinline__ u32x2 gather_g4(const PageSegs& s, int e) {
    const int k = (s.n[1] > 0 && e >= s.off[1]) ? 1 : 0;
    const int rel = e - s.off[k];
    const int n = s.n[k];
    u32x2 w = u32x2{0u, 0u};
    if (rel >= 0 && rel + 4 <= n) {
        w = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(s.g[k] + rel));
    } else if (rel >= 0 && rel < n) {
        const uint16_t* src = s.g[k] + rel;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (rel + j < n) w[j >> 1] |= (uint32_t)src[j] << (16 * (j & 1));
    }
    return w;
}

// bf16 parameters of page elements [e, e+4) written to the tenant tensor they belong to; elements
// of no tenant are dropped.
__device__ __forceinline__ void scatter_q4(const PageSegs& s, int e, u32x2 o) {
    const int k = (s.n[1] > 0 && e >= s.off[1]) ? 1 : 0;
    const int rel = e - s.off[k];
    const int n = s.n[k];
    if (rel >= 0 && rel + 4 <= n) {
        __builtin_nontemporal_store(o, reinterpret_cast<u32x2*>(s.q[k] + rel));
    } else if (rel >= 0 && rel < n) {
        uint16_t* dst = s.q[k] + rel;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (rel + j < n) dst[j] = (uint16_t)(o[j >> 1] >> (16 * (j & 1)));
    }
}

struct ReduceArgs {
    const uint16_t* g16;
    const PageSegs* segs;
    const int32_t* used;
    const int64_t* grad_pages;
    int64_t grad_first;
    int64_t list_offset;
    int64_t E;
    double* partials;
    uint32_t* nzflags;
    int32_t S;
};

// Per (page, slice): sum of squares in fp64 and OR of the magnitude bits of the slice's used
// gradient elements.  Slice 0 always writes (a zero for an empty page); other slices only when
// they hold used elements.  The fixed order (lane-sequential, wavefront butterfly, wave 0..3)
// makes the result independent of scheduling.
template <bool GATHER>
__global__ __launch_bounds__(kThreads) void apm_grad_reduce_kernel(ReduceArgs a) {
    const int64_t i = a.list_offset + blockIdx.y;
    const int64_t page = a.grad_pages ? a.grad_pages[i] : a.grad_first + i;
    const int used = a.used[page];
    const int start = blockIdx.x * kReduceTile;
    if (start >= used && blockIdx.x != 0) return;
    const int end = min(start + kReduceTile, used);
    const uint16_t* g = GATHER ? nullptr : a.g16 + page * a.E;
    PageSegs segs{};
    bool edge = false;  // gather only: this slice is not wholly inside one tenant
    if (GATHER) {
        segs = a.segs[i];
        const int k = (segs.n[1] > 0 && start >= segs.off[1]) ? 1 : 0;
        const int rel = start - segs.off[k];
        // Wholly inside tenant k, counted in whole 8-element vectors (the fast path below loads
        // 16 bytes at a time and must not read past the tensor's last element): address the
        // tensor like a page whose element 0 sits at g[k] - off[k].  A slice that holds a tensor's
        // ragged end takes the per-vector path, which reads that end element by element.
        const int span8 = ((end - start) + 7) & ~7;
        if (rel >= 0 && rel + span8 <= segs.n[k]) g = segs.g[k] - segs.off[k];
        else edge = true;
    }

    double acc0 = 0.0, acc1 = 0.0;
    uint32_t nz = 0;
    constexpr int U = APM_REDUCE_U;
    constexpr int kOuter = kReduceTile / (kThreads * 8 * U);
    static_assert(kOuter * kThreads * 8 * U == kReduceTile, "reduce tile must be a multiple of the unrolled span");
#pragma unroll 1
    for (int o = 0; o < kOuter; ++o) {
        const int e0 = start + o * (kThreads * 8 * U) + (int)threadIdx.x * 8;
        if (e0 - (int)threadIdx.x * 8 >= end) break;   // uniform: the whole span is beyond the extent
        u32x4 w[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * (kThreads * 8);
            w[u] = u32x4{0u, 0u, 0u, 0u};
            if (e < end) {
                if (GATHER && edge) w[u] = gather_g8(segs, e);
                else w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(g + e));
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * (kThreads * 8);
            if (e + 8 > end && e < end) {  // boundary vector: drop elements at or beyond the extent
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    uint32_t x = w[u][j];
                    if (e + 2 * j >= end) x = 0u;
                    else if (e + 2 * j + 1 >= end) x &= 0x0000FFFFu;
                    w[u][j] = x;
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t x = w[u][j];
                nz |= x & 0x7FFF7FFFu;
                const double lo = (double)bf16lo(x), hi = (double)bf16hi(x);
                acc0 = fma(lo, lo, acc0);
                acc1 = fma(hi, hi, acc1);
            }
        }
    }
    double acc = wave_sum_f64(acc0 + acc1);
    nz = wave_or_u32(nz);
    __shared__ double s_acc[kThreads / kWave];
    __shared__ uint32_t s_nz[kThreads / kWave];
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) {
        s_acc[wave] = acc;
        s_nz[wave] = nz;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = s_acc[0];
        uint32_t z = s_nz[0];
#pragma unroll
        for (int k = 1; k < kThreads / kWave; ++k) {
            t += s_acc[k];
            z |= s_nz[k];
        }
        a.partials[i * a.S + blockIdx.x] = t;
        a.nzflags[i * a.S + blockIdx.x] = z;
    }
}

struct FinalizeArgs {
    const int32_t* used;
    const int64_t* grad_pages;
    const int64_t* state_pages;
    int64_t grad_first;
    int64_t state_first;
    int64_t n_listed;
    const double* partials;
    const uint32_t* nzflags;
    int32_t S;
    int32_t skip_mode;
    double max_norm;
    PageMeta* meta;    // [n_listed]
    float* grad_norm;  // nullable
    uint8_t* skip_mask;  // nullable
    const int32_t* out_index;  // nullable: list position -> index into grad_norm / skip_mask
};

// One wavefront per listed page: combines the page's slice partials in a fixed order and turns
// them into the page's clip scale / skip decision and the optional outputs.
__global__ __launch_bounds__(kThreads) void apm_grad_finalize_kernel(FinalizeArgs a) {
    const int64_t i = (int64_t)blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
    if (i >= a.n_listed) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t page = a.grad_pages ? a.grad_pages[i] : a.grad_first + i;
    const int used = a.used[page];
    const int n_slices = max(1, (used + kReduceTile - 1) / kReduceTile);
    double s = 0.0;
    uint32_t nz = 0;
    for (int k = lane; k < n_slices; k += kWave) {
        s += a.partials[i * a.S + k];
        nz |= a.nzflags[i * a.S + k];
    }
    s = wave_sum_f64(s);
    nz = wave_or_u32(nz);
    if (lane != 0) return;
    const bool skip = a.skip_mode == APM_SKIP_UNTOUCHED && nz == 0u;
    const double norm = sqrt(s);
    float scale = 1.0f;
    if (a.max_norm > 0.0) {
        // min(1, c / (norm + 1e-6)) with plain IEEE propagation: an infinite norm gives 0, a NaN
        // norm a NaN scale (the comparison below is false for NaN), as the library optimizers do
        const double sc = a.max_norm / (norm + 1e-6);
        scale = sc > 1.0 ? 1.0f : (float)sc;
    }
    PageMeta pm;
    pm.used = used;
    pm.scale = skip ? -1.0f : scale;
    pm.gpage = page;
    pm.spage = a.state_pages ? a.state_pages[i] : a.state_first + i;
    pm.pad = 0;
    a.meta[i] = pm;
    const int64_t o = a.out_index ? (int64_t)a.out_index[i] : i;
    if (a.grad_norm) a.grad_norm[o] = skip ? 0.0f : (float)norm;
    if (a.skip_mask) a.skip_mask[o] = skip ? 1 : 0;
}

// No reduce pass: one thread per listed page fills its record with scale 1.
__global__ __launch_bounds__(kThreads) void apm_page_meta_kernel(FinalizeArgs a) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= a.n_listed) return;
    const int64_t page = a.grad_pages ? a.grad_pages[i] : a.grad_first + i;
    PageMeta pm;
    pm.used = a.used[page];
    pm.scale = 1.0f;
    pm.gpage = page;
    pm.spage = a.state_pages ? a.state_pages[i] : a.state_first + i;
    pm.pad = 0;
    a.meta[i] = pm;
}

struct UpdateArgs {
    float* p32;
    float* m32;
    float* v32;
    const uint16_t* g16;
    uint16_t* p16;
    const PageMeta* meta;  // per listed page
    const PageSegs* segs;  // per listed page (gather / scatter only)
    int64_t list_offset;
    int64_t E;
    float b1, omb1, b2, omb2, inv_sqrt_bc2, eps, step_size, lr_wd;
};

__device__ __forceinline__ void adamw_elem(float& p, float& m, float& v, float g, const UpdateArgs& a,
                                           float scale) {
    const float gs = g * scale;
    m = fmaf(a.b1, m, a.omb1 * gs);
    v = fmaf(a.b2, v, a.omb2 * (gs * gs));
#if APM_FAST_RCP_SQRT
    const float denom = fmaf(__builtin_amdgcn_sqrtf(v), a.inv_sqrt_bc2, a.eps);
    const float upd = m * __builtin_amdgcn_rcpf(denom);
#else
    const float denom = fmaf(sqrtf(v), a.inv_sqrt_bc2, a.eps);
    const float upd = m / denom;
#endif
    // p' = p - (lr wd p + (lr/bc1) m'/denom): the two small terms are summed first, so the only
    // rounding at the magnitude of p is the final subtraction (half an ulp per step).
    const float delta = fmaf(a.step_size, upd, a.lr_wd * p);
    p = p - delta;
}

constexpr int kUpdThreads = APM_UPDATE_THREADS;
constexpr int kUpdU = APM_UPDATE_U;
constexpr int kUpdTile = kUpdThreads * 4 * kUpdU;  // elements per workgroup

// The body of a slice.  EDGE_G / EDGE_Q: the slice is not wholly inside one tenant tensor, so g is
// gathered / p16 scattered lane by lane through the tenant descriptors; otherwise G and P16 are
// plain page-like pointers and the body is straight-line code (all loads issued back to back, one
// wait, all stores issued back to back).  The two forms are separate instantiations on purpose:
// with the per-lane paths as branches inside one body the compiler put a wait for all outstanding
// memory operations -- the stores of the previous vector included -- in front of every vector.
//
// FULL: every lane's kUpdU vectors lie inside the used extent (all slices of a page but its last),
// so no access is predicated and the whole body is one basic block.  That matters beyond the
// saved compares: on this target loads and stores share one counter, and at the entry of a basic
// block the compiler must assume the worst about what is outstanding -- with a predicate per
// vector, each vector's arithmetic began with a wait for every earlier memory operation, the
// previous vector's stores included, i.e. three extra store round trips per wavefront.
// Stores of the fp32 state: non-temporal, or -- WT, for state in host memory while other kernels
// run on the GPU -- written through at system scope.  A non-temporal store to host memory may rest
// in the L2 as a dirty line; the write-back that ends every kernel of any other stream then has
// to push it across PCIe, so those kernels pay for this kernel's writes.
template <bool WT>
__device__ __forceinline__ void store_state(f32x4 x, f32x4* q) {
    // Hand-written because no builtin takes a cache policy for a 128-bit global store; the wait
    // states keep the next instruction off the data registers, which a store of more than 64 bits
    // still reads right after issue (the compiler does that for its own stores, not for this one).
    if (WT) asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(q), "v"(x) : "memory");
    else __builtin_nontemporal_store(x, q);
}

template <bool EDGE_G, bool EDGE_Q, bool FULL, bool WT = false>
__device__ __forceinline__ void slice_body(const UpdateArgs& a, const PageSegs& segs, float scale, int nvec, int v0,
                                           f32x4* __restrict__ P, f32x4* __restrict__ M, f32x4* __restrict__ V,
                                           const u32x2* __restrict__ G_, u32x2* __restrict__ P16_) {
    // The tenant pointers come out of memory, so the compiler knows no address space for them and
    // would use flat accesses, which count against both memory counters and force full waits.
    // They are device (or pinned host) memory: say so.
    typedef const u32x2 __attribute__((address_space(1))) * GlobalIn;
    typedef u32x2 __attribute__((address_space(1))) * GlobalOut;
    const GlobalIn G = (GlobalIn)G_;
    const GlobalOut P16 = (GlobalOut)P16_;
    f32x4 p[kUpdU], m[kUpdU], v[kUpdU];
    u32x2 g[kUpdU];
#pragma unroll
    for (int u = 0; u < kUpdU; ++u) {
        const int vi = v0 + u * kUpdThreads;
        if (FULL || vi < nvec) {
            if (EDGE_G) g[u] = gather_g4(segs, vi << 2);
            else g[u] = __builtin_nontemporal_load(G + vi);
            p[u] = __builtin_nontemporal_load(P + vi);
            m[u] = __builtin_nontemporal_load(M + vi);
            v[u] = __builtin_nontemporal_load(V + vi);
        }
    }
    // all loads are issued before any arithmetic: without the barrier the scheduler, now that the
    // body is one block, sinks half of them between the vectors' arithmetic to save registers
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < kUpdU; ++u) {
        const int vi = v0 + u * kUpdThreads;
        if (FULL || vi < nvec) {
            const float gf[4] = {bf16lo(g[u][0]), bf16hi(g[u][0]), bf16lo(g[u][1]), bf16hi(g[u][1])};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float pj = p[u][j], mj = m[u][j], vj = v[u][j];
                adamw_elem(pj, mj, vj, gf[j], a, scale);
                p[u][j] = pj;
                m[u][j] = mj;
                v[u][j] = vj;
            }
            u32x2 o;
            o[0] = f32_to_bf16_rne(p[u][0]) | (f32_to_bf16_rne(p[u][1]) << 16);
            o[1] = f32_to_bf16_rne(p[u][2]) | (f32_to_bf16_rne(p[u][3]) << 16);
            store_state<WT>(p[u], P + vi);
            store_state<WT>(m[u], M + vi);
            store_state<WT>(v[u], V + vi);
            if (EDGE_Q) scatter_q4(segs, vi << 2, o);
            else __builtin_nontemporal_store(o, P16 + vi);
        }
    }
}

// Fused update of one slice (kUpdTile elements from `start`) of one page by one wavefront:
// 12 B + 2 B read and 12 B + 2 B written per element.  Each lane keeps kUpdU 128-bit vectors per
// fp32 class in flight; every wavefront-wide access is one contiguous 1 KiB (fp32) or 512 B (bf16)
// span.  GATHER / SCATTER: read g from / write p16 to the tenant tensors instead of the page
// classes.
template <bool GATHER, bool SCATTER, bool WT = false>
__device__ __forceinline__ void update_slice(const UpdateArgs& a, const PageSegs& segs, float scale,
                                             int used8, int64_t gpage, int64_t spage, int start, int lane) {
    f32x4* __restrict__ P = reinterpret_cast<f32x4*>(a.p32 + spage * a.E);
    f32x4* __restrict__ M = reinterpret_cast<f32x4*>(a.m32 + spage * a.E);
    f32x4* __restrict__ V = reinterpret_cast<f32x4*>(a.v32 + spage * a.E);
    const u32x2* __restrict__ G = GATHER ? nullptr : reinterpret_cast<const u32x2*>(a.g16 + gpage * a.E);
    u32x2* __restrict__ P16 = SCATTER ? nullptr : reinterpret_cast<u32x2*>(a.p16 + gpage * a.E);
    const int nvec = used8 >> 2;
    const int v0 = (start >> 2) + lane;
    if (GATHER || SCATTER) {
        const int k = (segs.n[1] > 0 && start >= segs.off[1]) ? 1 : 0;
        const int rel = start - segs.off[k];
        const int span = min(kUpdTile, used8 - start);
        // Wholly inside tenant k (the common case): address the tensor like a page whose element 0
        // sits at ptr - off[k]; the slice then runs the same code as the page-class path.
        if (rel >= 0 && rel + span <= segs.n[k]) {
            if (GATHER) G = reinterpret_cast<const u32x2*>(segs.g[k] - segs.off[k]);
            if (SCATTER) P16 = reinterpret_cast<u32x2*>(segs.q[k] - segs.off[k]);
        } else {
            slice_body<GATHER, SCATTER, false, WT>(a, segs, scale, nvec, v0, P, M, V, G, P16);
            return;
        }
    }
    if (start + kUpdTile <= used8) slice_body<false, false, true, WT>(a, segs, scale, nvec, v0, P, M, V, G, P16);
    else slice_body<false, false, false, WT>(a, segs, scale, nvec, v0, P, M, V, G, P16);
}

typedef long long i64x4 __attribute__((ext_vector_type(4)));
static_assert(sizeof(PageMeta) == sizeof(i64x4), "PageMeta must be 32 bytes");

// The HBM-resident form: grid.y walks the list positions, grid.x the slices (SLICES per
// workgroup) of a page.
template <bool GATHER, bool SCATTER, int SLICES>
__global__ __launch_bounds__(kUpdThreads) void apm_adamw_kernel(UpdateArgs a) {
    // Prologue: everything a workgroup needs about its page comes with one 32-byte scalar load
    // (plus the tenant descriptors in gather / scatter mode, fetched alongside).  A workgroup holds
    // a residency slot without memory traffic until this arrives, so the dependent-load chain is
    // kept to kernel arguments -> page record.
    const int64_t i = a.list_offset + blockIdx.y;
    const i64x4 raw = *reinterpret_cast<const i64x4*>(a.meta + i);  // one load for the whole record
    PageSegs segs{};
    if (GATHER || SCATTER) segs = a.segs[i];
#if APM_HOIST_LOADS
    // The exits below would let the compiler sink every scalar load that only the working path
    // needs (the tenant descriptors, the class base pointers) below them, which adds a third
    // dependent memory round trip to the prologue.  Naming the values as inputs of an empty asm
    // statement keeps those loads up here, in flight together with the page record.
    asm volatile("" ::"s"(a.p32), "s"(a.m32), "s"(a.v32), "s"(a.g16), "s"(a.p16), "s"(a.E));
    if (GATHER || SCATTER)
        asm volatile("" ::"s"(segs.off[0]), "s"(segs.off[1]), "s"(segs.n[0]), "s"(segs.n[1]), "s"(segs.g[0]),
                     "s"(segs.g[1]), "s"(segs.q[0]), "s"(segs.q[1]));
#endif
    const float scale = __uint_as_float((uint32_t)((uint64_t)raw[0] >> 32));
    const int used8 = ((int32_t)(uint32_t)raw[0] + 7) & ~7;
    // (Folding the two exits below into the lane predicate, so that all scalar loads of the
    // prologue issue together, measured 2-3 % slower on the 1.3 B workload and 3 % faster on the
    // fragmented 124 M one; the early exits stay.)
    if (scale < 0.0f) return;  // a skipped page
#pragma unroll 1
    for (int it = 0; it < SLICES; ++it) {
        const int start = ((int)blockIdx.x * SLICES + it) * kUpdTile;
        if (start >= used8) return;  // beyond the extent
        update_slice<GATHER, SCATTER>(a, segs, scale, used8, raw[1], raw[2], start, (int)threadIdx.x);
    }
}

// The form for fp32 classes that live in pinned host memory and are read and written across
// PCIe by the kernel itself: a fixed number of wavefronts walks all (position, slice) items of
// `count` list positions with `nx` slices each, consecutive wavefronts taking consecutive slices.
// The link needs only some hundred KiB in flight, so a few dozen wavefronts saturate it.  The
// launch chooses how many of them share a workgroup (and with it a CU): one per workgroup gives
// the highest transfer rate; packed 8 or 16 to a workgroup they occupy few CUs, which matters
// beside kernels whose workgroups need a CU's whole register file or LDS (dense matrix
// products), because a wavefront that lives as long as the whole transfer keeps those off its CU.
constexpr int kStrideMaxThreads = 1024;

template <bool GATHER, bool SCATTER, bool WT>
__global__ __launch_bounds__(kStrideMaxThreads) void apm_adamw_stride_kernel(UpdateArgs a, int64_t count, int nx,
                                                                             int n_workers) {
    const int lane = (int)threadIdx.x & (kWave - 1);
    const int waves_per_wg = (int)blockDim.x / kWave;
    const int worker = (int)blockIdx.x * waves_per_wg + __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
    if (worker >= n_workers) return;
    const int64_t n_items = count * nx;
#pragma unroll 1
    for (int64_t w = worker; w < n_items; w += n_workers) {
        const int64_t i = a.list_offset + w / nx;
        const int start = (int)(w % nx) * kUpdTile;
        const i64x4 raw = *reinterpret_cast<const i64x4*>(a.meta + i);
        const float scale = __uint_as_float((uint32_t)((uint64_t)raw[0] >> 32));
        const int used8 = ((int32_t)(uint32_t)raw[0] + 7) & ~7;
        if (scale < 0.0f || start >= used8) continue;
        PageSegs segs{};
        if (GATHER || SCATTER) segs = a.segs[i];
        update_slice<GATHER, SCATTER, WT>(a, segs, scale, used8, raw[1], raw[2], start, lane);
    }
}

struct AccumArgs {
    uint16_t* acc;        // buffered gradient g' (page layout)
    const uint16_t* g16;  // incoming gradient (page layout)
    const int32_t* used;
    const int64_t* pages;
    int64_t first;
    int64_t list_offset;
    int64_t E;
};

// g' <- bf16_rne(fp32(g') + fp32(g)) over the used extent of each listed page (Alg. 2, buffering
// thread: "accumulate buffered gradients").  6 B/element, HBM-bound; same slicing as the reduce.
__global__ __launch_bounds__(kThreads) void apm_grad_accum_kernel(AccumArgs a) {
    const int64_t i = a.list_offset + blockIdx.y;
    const int64_t page = a.pages ? a.pages[i] : a.first + i;
    const int used8 = (a.used[page] + 7) & ~7;
    const int start = blockIdx.x * kReduceTile;
    if (start >= used8) return;
    const int end = min(start + kReduceTile, used8);
    u32x4* acc = reinterpret_cast<u32x4*>(a.acc + page * a.E);
    const u32x4* g = reinterpret_cast<const u32x4*>(a.g16 + page * a.E);
    constexpr int U = 4;
#pragma unroll 1
    for (int e0 = start + (int)threadIdx.x * 8; e0 - (int)threadIdx.x * 8 < end; e0 += kThreads * 8 * U) {
        u32x4 x[U], y[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * (kThreads * 8);
            if (e < end) {
                x[u] = __builtin_nontemporal_load(acc + (e >> 3));
                y[u] = __builtin_nontemporal_load(g + (e >> 3));
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * (kThreads * 8);
            if (e < end) {
                u32x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float lo = bf16lo(x[u][j]) + bf16lo(y[u][j]);
                    const float hi = bf16hi(x[u][j]) + bf16hi(y[u][j]);
                    o[j] = f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
                }
                __builtin_nontemporal_store(o, acc + (e >> 3));
            }
        }
    }
}

constexpr int kMaxGridY = 65535;

}  // namespace

hipError_t launch_grad_accum(uint16_t* acc, const uint16_t* g16, const int32_t* used,
                             const int64_t* d_pages, int64_t first, int64_t n_listed, int64_t E,
                             hipStream_t s) {
    AccumArgs a{acc, g16, used, d_pages, first, 0, E};
    const unsigned nx = (unsigned)((E + kReduceTile - 1) / kReduceTile);
    for (int64_t off = 0; off < n_listed; off += kMaxGridY) {
        const int64_t ny = n_listed - off < kMaxGridY ? n_listed - off : kMaxGridY;
        a.list_offset = off;
        hipLaunchKernelGGL(apm_grad_accum_kernel, dim3(nx, (unsigned)ny), dim3(kThreads), 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

namespace {
// Calls f(first list position, pages, largest used extent) for every launch of a pass: per extent
// class, in pieces of at most kMaxGridY pages.
template <class F>
hipError_t for_each_launch(const AdamwLaunch& L, F&& f) {
    const ExtentClass all{0, L.n_listed, L.E};
    const ExtentClass* c = L.n_cls > 0 ? L.cls : &all;
    const int n = L.n_cls > 0 ? L.n_cls : 1;
    for (int k = 0; k < n; ++k) {
        for (int64_t off = 0; off < c[k].count; off += kMaxGridY) {
            const int64_t ny = c[k].count - off < kMaxGridY ? c[k].count - off : kMaxGridY;
            f(c[k].begin + off, ny, c[k].max_used > 0 ? c[k].max_used : 1);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}
}  // namespace

hipError_t launch_grad_reduce(const AdamwLaunch& L, hipStream_t s) {
    ReduceArgs a{L.g16, L.segs, L.used, L.grad_pages, L.grad_first, 0, L.E, L.partials, L.nzflags, L.S};
    hipError_t e = for_each_launch(L, [&](int64_t begin, int64_t ny, int64_t max_used) {
        a.list_offset = begin;
        const dim3 grid((unsigned)((max_used + kReduceTile - 1) / kReduceTile), (unsigned)ny);
        if (L.gather) hipLaunchKernelGGL(apm_grad_reduce_kernel<true>, grid, dim3(kThreads), 0, s, a);
        else hipLaunchKernelGGL(apm_grad_reduce_kernel<false>, grid, dim3(kThreads), 0, s, a);
    });
    if (e != hipSuccess) return e;
    FinalizeArgs f{L.used, L.grad_pages, L.state_pages, L.grad_first, L.state_first, L.n_listed,
                   L.partials, L.nzflags, L.S, L.skip_mode, L.max_norm, L.meta, L.grad_norm, L.skip_mask,
                   L.out_index};
    const int per_wg = kThreads / kWave;
    hipLaunchKernelGGL(apm_grad_finalize_kernel, dim3((unsigned)((L.n_listed + per_wg - 1) / per_wg)),
                       dim3(kThreads), 0, s, f);
    return hipGetLastError();
}

hipError_t launch_prepare(const AdamwLaunch& L, hipStream_t s) {
    FinalizeArgs f{L.used, L.grad_pages, L.state_pages, L.grad_first, L.state_first, L.n_listed,
                   nullptr, nullptr, L.S, L.skip_mode, 0.0, L.meta, nullptr, nullptr, nullptr};
    hipLaunchKernelGGL(apm_page_meta_kernel, dim3((unsigned)((L.n_listed + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, s, f);
    return hipGetLastError();
}

hipError_t launch_adamw(const AdamwLaunch& L, hipStream_t s) {
    UpdateArgs a{};
    a.p32 = L.p32; a.m32 = L.m32; a.v32 = L.v32; a.g16 = L.g16; a.p16 = L.p16;
    a.segs = L.segs;
    a.meta = L.meta;
    a.E = L.E;
    a.b1 = L.b1; a.omb1 = L.omb1; a.b2 = L.b2; a.omb2 = L.omb2;
    a.inv_sqrt_bc2 = L.inv_sqrt_bc2; a.eps = L.eps; a.step_size = L.step_size; a.lr_wd = L.lr_wd;
    if (L.stride_wavefronts > 0) {
        return for_each_launch(L, [&](int64_t begin, int64_t ny, int64_t max_used) {
            a.list_offset = begin;
            const int nx = (int)((max_used + kUpdTile - 1) / kUpdTile);
            const int64_t items = ny * nx;
            const int workers = (int)(items < L.stride_wavefronts ? items : L.stride_wavefronts);
            const int per_wg = L.stride_waves_per_wg >= 1 && L.stride_waves_per_wg <= kStrideMaxThreads / kWave ? L.stride_waves_per_wg : 1;
            const dim3 grid((unsigned)((workers + per_wg - 1) / per_wg)), block((unsigned)(per_wg * kWave));
#define APM_LAUNCH_STRIDE(G, Q)                                                                                       \
    do {                                                                                                             \
        if (L.host_write_through) hipLaunchKernelGGL((apm_adamw_stride_kernel<G, Q, true>), grid, block, 0, s, a, ny, nx, workers); \
        else hipLaunchKernelGGL((apm_adamw_stride_kernel<G, Q, false>), grid, block, 0, s, a, ny, nx, workers);       \
    } while (0)
            if (L.gather && L.scatter) APM_LAUNCH_STRIDE(true, true);
            else if (L.gather) APM_LAUNCH_STRIDE(true, false);
            else if (L.scatter) APM_LAUNCH_STRIDE(false, true);
            else APM_LAUNCH_STRIDE(false, false);
#undef APM_LAUNCH_STRIDE
        });
    }
    const bool may_skip = L.partials && L.skip_mode == APM_SKIP_UNTOUCHED;
    const int64_t wg_span = (int64_t)kUpdTile * (may_skip ? APM_UPDATE_SLICES_SKIP : 1);
    return for_each_launch(L, [&](int64_t begin, int64_t ny, int64_t max_used) {
        a.list_offset = begin;
        const dim3 grid((unsigned)((max_used + wg_span - 1) / wg_span), (unsigned)ny), block(kUpdThreads);
#define APM_LAUNCH_UPDATE(G, Q)                                                                         \
    do {                                                                                               \
        if (may_skip) hipLaunchKernelGGL((apm_adamw_kernel<G, Q, APM_UPDATE_SLICES_SKIP>), grid, block, APM_UPDATE_LDS, s, a); \
        else hipLaunchKernelGGL((apm_adamw_kernel<G, Q, 1>), grid, block, APM_UPDATE_LDS, s, a);       \
    } while (0)
        if (L.gather && L.scatter) APM_LAUNCH_UPDATE(true, true);
        else if (L.gather) APM_LAUNCH_UPDATE(true, false);
        else if (L.scatter) APM_LAUNCH_UPDATE(false, true);
        else APM_LAUNCH_UPDATE(false, false);
#undef APM_LAUNCH_UPDATE
    });
}

}  // namespace apm
