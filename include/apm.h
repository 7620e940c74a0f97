/*
 * apm — page-granular mixed-precision AdamW for MI355X (gfx950).  C ABI.
 *
 * The library implements, on one GPU, the optimizer-update hot path of Angel-PTM
 * (arXiv 2303.02868): model states live in fixed-size pages (Sec. 4.1), the update of the FP32
 * master parameter / momentum / variance from 16-bit gradients and the cast back to 16-bit
 * parameters run page by page (Alg. 2; Sec. 4.3, last paragraph), pages move between pinned host
 * memory and HBM asynchronously (Sec. 5 "Allocator") overlapped with the update (Sec. 4.2), and a
 * one-step-stale variant decouples gradient production from the update (Sec. 4.3, Alg. 2).
 *
 * Conventions
 *   - Every function returns an apm_status (0 = ok, negative = error) unless stated; nothing
 *     throws or aborts.  On error, outputs are untouched and apm_last_error() describes the cause.
 *   - "device pointer" = HBM or pinned-host memory the GPU can address; "host pointer" = ordinary
 *     host memory read or written by the CPU during the call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  GPU work is enqueued
 *     on it and the call returns without waiting; only argument and capacity errors are reported
 *     synchronously.
 *   - A pool and everything it owns belong to one HIP device.  Calls on one pool must be issued
 *     from one thread at a time and, unless stated, be ordered by the caller's streams: the pool's
 *     internal scratch is shared by its calls.
 *   - Element counts are in elements, never bytes, unless the name says bytes.
 */
#ifndef APM_H
#define APM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct apm_pool apm_pool;
typedef struct apm_streamer apm_streamer;
typedef struct apm_tiered apm_tiered;

enum apm_status {
    APM_OK = 0,
    APM_EINVAL = -1,  /* bad argument */
    APM_ENOMEM = -2,  /* allocation failed or pool capacity exceeded */
    APM_ERANGE = -3,  /* page / state index out of range */
    APM_EDEVICE = -4, /* HIP runtime error or wrong device kind */
    APM_ESTATE = -5   /* call not valid in the pool's current state */
};

/* Where a pool's pages live, numbered like the paper's device map {0: GPU, 1: CPU, 2: SSD} (Page
 * listing, Sec. 4.1).  A FILE pool keeps each state class in one file (apm_file_pool_create). */
enum apm_device { APM_DEV_GPU = 0, APM_DEV_HOST = 1, APM_DEV_FILE = 2 };

enum apm_dtype { APM_F32 = 0, APM_BF16 = 1 };

/* The five state classes of a page group (Alg. 2 inputs): FP32 master parameter, momentum,
 * variance; 16-bit gradient; 16-bit (buffered) parameter.  16-bit means bf16 (Sec. 6.1). */
enum apm_state { APM_P32 = 0, APM_M32 = 1, APM_V32 = 2, APM_G16 = 3, APM_P16 = 4, APM_N_STATES = 5 };

enum apm_skip_mode {
    APM_SKIP_NONE = 0,     /* every listed page is updated; zero gradients are ordinary gradients */
    APM_SKIP_UNTOUCHED = 1 /* a page whose used gradient elements are all +-0 is left bit-identical */
};

enum apm_pool_flags {
    APM_POOL_NO_ZERO = 1u, /* do not zero-fill at creation; the caller guarantees that unused page
                              elements (padding, alignment gaps) are zero in every state class.
                              FILE pools: existing files keep their contents */
    APM_POOL_FILE_DIRECT = 2u /* FILE pools: unbuffered I/O (O_DIRECT), bypassing the page cache */
};

/*
 * Pool description.  Page group k of a pool is the element range [k*E, (k+1)*E) of each state
 * class the pool stores; class s is one contiguous region of n_pages*E elements (fp32 classes
 * 4 B/element, bf16 classes 2 B/element), so consecutive pages are contiguous in memory.
 * With E = 1048576 an fp32 page is the paper's 4 MB page (Sec. 4.1 "Optimal Page Size").
 */
typedef struct {
    int32_t device;     /* apm_device */
    int32_t hip_device; /* HIP device ordinal that owns / addresses the pool */
    int64_t page_elems; /* E > 0, a multiple of 8 */
    int64_t n_pages;    /* capacity in page groups, > 0, at most 2^31 - 1 */
    uint32_t state_mask; /* bit s set = the pool stores state class s */
    uint32_t flags;      /* apm_pool_flags */
    /* base[s] != NULL: caller-owned region for class s (n_pages*E elements, 16-byte aligned,
     * HBM for a GPU pool, pinned host memory for a HOST pool); it must outlive the pool.
     * base[s] == NULL: the library allocates (hipMalloc / hipHostMalloc) and frees it. */
    void* base[APM_N_STATES];
} apm_pool_desc;

/* A caller-owned contiguous tensor.  `data` is a device pointer (see Conventions) of `numel`
 * elements of `dtype`, or NULL where a call only needs the size.  `id` is the caller's tensor id,
 * recorded in the page table (Tensor listing, Sec. 4.1). */
typedef struct {
    int64_t id;
    int32_t dtype; /* apm_dtype */
    int32_t reserved;
    int64_t numel;
    void* data;
} apm_tensor;

/* One contiguous piece of a tensor inside one page: elements [tensor_off, tensor_off+n) of tensor
 * number `tensor` (its index in the list) sit at [page_off, page_off+n) of page `page`. */
typedef struct {
    int64_t tensor, tensor_off, page, page_off, n;
} apm_segment;

/* Page-table entry, after the Page listing of Sec. 4.1 (sizes in elements of the page group). */
typedef struct {
    int64_t total_elems;     /* E */
    int64_t used_elems;      /* end offset of the last occupied element */
    int64_t available_elems; /* E - used_elems */
    int32_t device;          /* apm_device of the pool */
    int32_t n_tensors;       /* 0, 1 or 2 */
    int64_t tensor_id[2];    /* caller ids of the tenants (-1 = none) */
    int64_t tensor_elems[2]; /* elements each tenant occupies in this page */
} apm_page_info;

/* Optimizer hyper-parameters, as doubles; the library derives every step-dependent scalar in
 * double and rounds it to fp32 once.  max_grad_norm <= 0 switches per-page clipping off. */
typedef struct {
    double lr, beta1, beta2, eps, weight_decay, max_grad_norm;
    int32_t skip_mode; /* apm_skip_mode */
    int32_t reserved;
} apm_hyper;

/* ---- errors ------------------------------------------------------------------------------ */

/* Message of the calling thread's last failed call (library-owned, valid until the thread's next
 * failing call); "" if none. */
const char* apm_last_error(void);

/* ---- packing plan (host only; no GPU is touched) ------------------------------------------- */

/*
 * Deterministic layout of a ragged tensor list in pages of E elements (Sec. 4.1: at most two
 * tensors per page; a tensor smaller than a page takes a page of its own).  Tensors are placed in
 * list order; numel == 0 takes no page; 0 < numel < E takes a fresh page at offset 0 that admits
 * no second tenant; numel >= E starts in the open page if there is one (a page with one tenant and
 * room left after rounding its used extent up to 8 elements), else in a fresh page, continues
 * through fresh pages, and leaves its partly filled last page open.
 *
 * numels: host pointer, n entries >= 0.  segs: host pointer, capacity *n_segs on entry, count on
 * return (NULL with *n_segs == 0 to query the count only).  n_pages, fragmentation
 * (= 1 - sum(numel) / (n_pages*E)) : host pointers, nullable.
 * Errors: APM_EINVAL (bad E, negative numel, NULL n_segs), APM_ENOMEM (*n_segs too small; the
 * needed count is still returned in *n_segs).
 */
int apm_pack_plan(int64_t page_elems, const int64_t* numels, int64_t n, apm_segment* segs,
                  int64_t* n_segs, int64_t* n_pages, double* fragmentation);

/* ---- pool and page table (Sec. 4.1 Page; Sec. 5 "Allocator": pre-allocated memory cut into
 *      fixed-size pages) --------------------------------------------------------------------- */

/* Creates a pool.  *out is written only on success.  Every region is zero-filled (synchronously)
 * unless APM_POOL_NO_ZERO is set.  Errors: APM_EINVAL, APM_ENOMEM, APM_EDEVICE. */
int apm_pool_create(apm_pool** out, const apm_pool_desc* desc);

/* Waits for the pool's internal streams, frees what the library allocated.  NULL is accepted. */
int apm_pool_destroy(apm_pool* pool);

/* Number of pages the installed layout occupies (0 before any layout). */
int64_t apm_pool_pages_in_use(const apm_pool* pool);

/* Page-table entry of `page` (host pointer out).  APM_ERANGE if page >= capacity. */
int apm_pool_page_info(const apm_pool* pool, int64_t page, apm_page_info* out);

/* Device pointer of the first element of `page` in class `state`, or NULL (class not stored, page
 * out of range). */
void* apm_pool_state_ptr(const apm_pool* pool, int state, int64_t page);

/*
 * Installs the layout of a tensor list (apm_pack_plan's rule) in the pool's page table without
 * copying data — tensors are then "born" in pages.  Only id and numel of each tensor are read.
 * Re-installing a different layout zero-fills every class the pool stores first (on `stream`).
 * Outputs as in apm_pack_plan.  Errors: APM_ENOMEM if the layout needs more pages than the pool
 * has.
 */
int apm_pool_set_layout(apm_pool* pool, const apm_tensor* tensors, int64_t n, apm_segment* segs,
                        int64_t* n_segs, int64_t* n_pages, double* fragmentation, void* stream);

/* ---- kernel timing (measurement aid) -------------------------------------------------------- */

enum apm_kernel_class { APM_K_REDUCE = 0, APM_K_UPDATE = 1, APM_K_SEGCOPY = 2, APM_N_KERNEL_CLASSES = 3 };

/* While enabled, every kernel the pool's calls launch (apm_page_adamw_step, apm_pack_tensors,
 * apm_unpack) is bracketed by a pair of HIP events on the stream it is launched on. */
int apm_pool_set_timing(apm_pool* pool, int enable);

/* Waits for the recorded events, adds the elapsed milliseconds per kernel class into
 * ms[APM_N_KERNEL_CLASSES] and the launch counts into launches[APM_N_KERNEL_CLASSES] (host
 * pointers, overwritten), and forgets the events. */
int apm_pool_read_timing(apm_pool* pool, double* ms, int64_t* launches);

/* ---- pack / unpack (gather / scatter kernels; the Tensor listing's merge is apm_unpack) ---- */

/*
 * Copies the tensors' elements, bit for bit, into class `state` of the pool's pages.  If the pool
 * has no layout yet the list's layout is installed first; otherwise the list must have the same
 * numels as the installed layout (APM_ESTATE if not).  tensors[i].dtype must match the class
 * (APM_F32 for P32/M32/V32, APM_BF16 for G16/P16) and tensors[i].data must be a device pointer
 * (any alignment; 16-byte alignment takes the fast path).  Padding is not written: it stays zero.
 * Outputs as in apm_pack_plan.  Asynchronous on `stream`.
 */
int apm_pack_tensors(apm_pool* pool, int state, const apm_tensor* tensors, int64_t n,
                     apm_segment* segs, int64_t* n_segs, int64_t* n_pages, double* fragmentation,
                     void* stream);

/* Inverse of apm_pack_tensors: scatters class `state` of the pages back into the contiguous
 * tensors dst[i].data.  The list must match the installed layout.  Asynchronous on `stream`. */
int apm_unpack(apm_pool* pool, int state, const apm_tensor* dst, int64_t n, void* stream);

/* ---- the update (Alg. 2 "Update p32, m32, v32 via g16", "p'16 <- cast(p32)") -------------- */

/*
 * One AdamW step on the listed pages of a GPU pool that stores all five classes.
 * For each listed page k with used extent n_k, with t = step (1-based, global):
 *   nz = any used gradient element with non-zero magnitude bits; if skip_mode is
 *   APM_SKIP_UNTOUCHED and !nz: skip_mask = 1, grad_norm = 0, page untouched.  Otherwise
 *   norm = sqrt(sum g^2) over the used elements (fp64 accumulation, fixed order),
 *   s = max_grad_norm > 0 ? min(1, max_grad_norm / (norm + 1e-6)) : 1,  g^ = s*g,
 *   m' = b1 m + (1-b1) g^;  v' = b2 v + (1-b2) g^2;
 *   p' = p (1 - lr wd) - lr (m'/(1-b1^t)) / (sqrt(v'/(1-b2^t)) + eps);   p16' = bf16_rne(p').
 * Arithmetic is fp32 with correctly rounded divide and square root; p' is evaluated as
 * p - (lr wd p + (lr/(1-b1^t)) m'/denom) so that it is rounded once at the magnitude of p.
 * Non-finite gradients get no special treatment (IEEE propagation: an infinite norm gives s = 0,
 * a NaN norm s = NaN).
 *
 * pages: host pointer to n_pages distinct page indices, or NULL = pages [0, n_pages).
 * grad_norm (float[n_pages]) and skip_mask (uint8_t[n_pages]): device pointers (or pinned host
 * memory, which the GPU addresses as well), nullable, indexed like `pages`, written by the kernel.
 * Errors: APM_EINVAL (step < 1, bad hyper-parameters, NULL hyper, a page listed twice),
 * APM_ERANGE (page index), APM_ESTATE (pool lacks a class), APM_EDEVICE.
 */
int apm_page_adamw_step(apm_pool* pool, const int64_t* pages, int64_t n_pages, int64_t step,
                        const apm_hyper* hyper, float* grad_norm, uint8_t* skip_mask,
                        void* stream);

/*
 * The same step with the gather and/or scatter fused into the kernels: gradients are read straight
 * from the caller's contiguous bf16 tensors (grad_tensors != NULL; the G16 class is not touched
 * and need not be stored) and the bf16 parameters are written straight into the caller's
 * contiguous bf16 tensors (p16_tensors != NULL; the P16 class is not touched).  This removes the
 * pack / unpack passes over 16-bit data (8 B/element of HBM traffic) from a training step; the
 * result is bit-identical to apm_pack_tensors(G16) + apm_page_adamw_step + apm_unpack(P16).
 * Each list must have the numels of the installed layout (APM_ESTATE otherwise), dtype APM_BF16
 * and 16-byte aligned device pointers (APM_EINVAL otherwise); either list may be NULL.
 * Listed pages must be pages the layout uses.
 */
int apm_page_adamw_step_fused(apm_pool* pool, const int64_t* pages, int64_t n_pages, int64_t step,
                              const apm_hyper* hyper, const apm_tensor* grad_tensors,
                              const apm_tensor* p16_tensors, int64_t n_tensors, float* grad_norm,
                              uint8_t* skip_mask, void* stream);

/*
 * apm_page_adamw_step for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same kernels and bit-identical results for the pages
 * [0, n_pages) of a GPU pool that stores all five classes (no page list; every page is launched
 * with a full page's grid, so nearly empty pages cost idle workgroups here).  The per-page scratch
 * of the reduce and update kernels (page records, per-slice sums of squares and non-zero flags)
 * lives in a fixed device array of apm_noalloc_scratch_bytes() bytes that the library holds on
 * every GPU it runs on until the process ends, instead of buffers the pool allocates on first use;
 * the call performs no hipMalloc / hipFree, creates no events or streams and allocates no host
 * memory (apm_pool_set_timing does not cover it).  The array's device address is resolved on the
 * first call on each device.
 * All calls on one GPU share that array and it keeps the last call's contents (every entry a call
 * reads it has written before, nothing needs clearing): calls that overlap on one GPU -- on
 * different streams, or from different pools -- race; order them on one stream or with events.
 * Errors: as apm_page_adamw_step; APM_ERANGE if n_pages exceeds apm_noalloc_max_pages(page_elems)
 * (the scratch holds 32 + 12 * ceil(page_elems / 16384) bytes per page: 5241 pages of 2^20
 * elements); nothing is enqueued then.
 */
int apm_page_adamw_step_noalloc(apm_pool* pool, int64_t n_pages, int64_t step,
                                const apm_hyper* hyper, float* grad_norm, uint8_t* skip_mask,
                                void* stream);
size_t apm_noalloc_scratch_bytes(void);
int64_t apm_noalloc_max_pages(int64_t page_elems);

/* ---- page movement (Page listing: move; Sec. 5 "Allocator": asynchronous GPU-CPU copies) --- */

/*
 * Copies class `state` of n_pages consecutive pages, src_page.. of `src` to dst_page.. of `dst`
 * (one asynchronous copy; H2D, D2H, D2D or H2H according to the pools' devices).  Both pools
 * must have the same page_elems and store the class.  Page-table entries are not copied.
 */
int apm_page_copy_async(apm_pool* dst, int64_t dst_page, apm_pool* src, int64_t src_page,
                        int64_t n_pages, int state, void* stream);

/* ---- streamed update: FP32 states in pinned host pages, updated page by page across PCIe
 *      (Sec. 4.2: overlap movement with computation, scheduled per page) -------------------- */

/*
 * host:   HOST pool storing P32, M32, V32 (the layout is taken from `dev`); it must hold every
 *         page in use unless apm_streamer_set_host_first_page says otherwise (checked per step).
 * dev:    GPU pool storing G16 and P16 for the same pages, with an installed layout.
 * batch_pages: pages moved and updated per pipeline stage of the staged mode (>= 1).
 * n_slots: staging slots in HBM for the staged mode (>= 2); each holds batch_pages pages of the
 *          three fp32 classes.
 * The streamer starts in APM_STREAM_DIRECT if the GPU can address the host pool's memory (pinned
 * memory: always), else in APM_STREAM_STAGED_DMA; see apm_streamer_set_mode.
 */
int apm_streamer_create(apm_streamer** out, apm_pool* host, apm_pool* dev, int64_t batch_pages,
                        int n_slots);
int apm_streamer_destroy(apm_streamer* s);

/*
 * How the fp32 pages cross PCIe (Sec. 4.2 leaves the mechanism open):
 *   APM_STREAM_DIRECT: no copies and no staging; the update kernel itself reads p, m, v from the
 *     pinned host pages and writes them back, with `direct_wavefronts` wavefronts (0 = 48, which
 *     saturates the link) of which `wavefronts_per_workgroup` (0 = 1, at most 16) share a
 *     workgroup and so a CU.  One per workgroup moves data fastest; more per workgroup occupy
 *     fewer CUs for the duration of the step, which disturbs concurrent kernels of the caller
 *     less (measured beside dense matrix products: 128 wavefronts, 16 per workgroup).
 *   APM_STREAM_STAGED: the double-buffered pipeline through HBM staging slots.  While batch b is
 *     updated in its slot, ONE copy kernel of the library (direct_wavefronts wavefronts, as above)
 *     brings batch b+1 from its host pages into the next slot and takes batch b-1 from the
 *     previous slot back to its host pages, both directions at once; with two slots the two
 *     directions are two kernels, one after the other.  A batch here is at most batch_pages
 *     pages: the batches are cut so that each holds about as many used elements as the emptiest
 *     run of batch_pages pages (an exchange lasts as long as its longer direction, and the kernel
 *     moves used extents only).  One copy stream and one compute stream;
 *     streams that share a hardware queue would run the update behind each copy kernel, so the
 *     copy stream is chosen, when the mode is first selected, by timing a pair of short kernels
 *     on each of a few candidates (about a millisecond each; synchronises the device).
 *     The staging memory is allocated when a staged mode is first selected.
 *   APM_STREAM_STAGED_DMA: the same slot ring moved by the runtime's asynchronous copies:
 *     copy-in / update / copy-out on three streams.  Which stream pairs overlap a host-to-device
 *     with a device-to-host copy depends on the runtime, so when this mode is first selected
 *     short concurrent copies are timed on a few candidate streams (the default stream among
 *     them) and the best pair is kept; this takes some tens of milliseconds and synchronises the
 *     device.  The only mode for host memory the GPU cannot address.
 * All modes give bit-identical results.  Takes effect from the next apm_streamer_step.
 * apm_streamer_get_mode returns the current mode (or a negative status).
 */
enum apm_stream_mode { APM_STREAM_STAGED = 0, APM_STREAM_DIRECT = 1, APM_STREAM_STAGED_DMA = 2 };
int apm_streamer_set_mode(apm_streamer* s, int mode, int direct_wavefronts,
                          int wavefronts_per_workgroup);
int apm_streamer_get_mode(const apm_streamer* s);

/*
 * One AdamW step over all pages in use.  Staged modes: for batch b, the copy-in of batch b+1 and
 * the copy-out of batch b-1 run beside update(b) on the compute stream, ordered by events.
 * Direct mode: one reduce pass and one update kernel on the compute stream.
 * The work starts after everything enqueued on `stream` so far, and `stream` is made to wait for
 * the step's completion; the host does not block.  grad_norm / skip_mask as in
 * apm_page_adamw_step (device pointers, one entry per page in use, nullable).
 */
int apm_streamer_step(apm_streamer* s, int64_t step, const apm_hyper* hyper, float* grad_norm,
                      uint8_t* skip_mask, void* stream);

/*
 * How the kernels that write the host pool (the direct mode's update kernel, the staged mode's and
 * the scheduled step's copy kernel) store: non-temporal (on = 0, the default: fastest when nothing
 * else runs on the GPU) or written through at system scope (on != 0).  A non-temporal store to host
 * memory may rest in the GPU's L2 as a dirty line; the write-back at the end of every kernel of any
 * other stream then has to push such lines across PCIe, so kernels that run beside the update are
 * stretched by its writes (measured: elementwise kernels beside the outbound half of the staged
 * pipeline ran 150 ms longer per 290 ms of traffic, beside written-through stores 10 ms).  Written
 * through, the step alone is about a tenth slower.  Meant for the one-step-stale forms, whose
 * update runs beside the caller's kernels.  Results are bit-identical.  Takes effect from the next
 * step.
 */
int apm_streamer_set_host_write_through(apm_streamer* s, int on);

/* GB/s the staged-DMA mode's stream calibration measured on 32 MiB copies (zeros before it ran):
 * copy-in alone, copy-out alone, and each way with both running on the chosen pair (host
 * pointers, nullable). */
int apm_streamer_probe_rates(const apm_streamer* s, double* h2d, double* d2h, double* duplex_each_way);

/*
 * Mixed residency (the GPU cache of optimizer states, Sec. 4.2): pages [0, n_resident) keep their
 * fp32 classes in `cache` (a GPU pool storing P32, M32, V32, same page size; its page k is model
 * page k) and are updated in place; only pages [n_resident, N) are streamed from the host pool.
 * Moving a page between the tiers is the caller's apm_page_copy_async between `cache` and the
 * host pool, done between steps.  cache == NULL or n_resident == 0 switches the cache off.
 */
int apm_streamer_set_cache(apm_streamer* s, apm_pool* cache, int64_t n_resident);

/*
 * Sizing the cache from the memory that is free now (Sec. 4.2: the cache size is decided per
 * model so that training does not run out of GPU memory): *out = how many of n_pages pages'
 * fp32 classes (12 * page_elems bytes each) fit into the device's free memory minus
 * reserve_bytes, at most n_pages.  Call it after the model's other GPU allocations.
 */
int apm_cache_pages_that_fit(int hip_device, int64_t page_elems, int64_t n_pages,
                             size_t reserve_bytes, int64_t* out);

/*
 * With a cache, the host pool need not hold the resident pages: after this call page j of the host
 * pool is model page first_model_page + j (default 0), so a host pool of N - first_model_page
 * pages serves a model of N pages whose first n_resident >= first_model_page pages are cached --
 * the way to run a model whose fp32 state exceeds what the machine can pin.  Checked at each step
 * (APM_ESTATE if pages are covered by neither pool or the host pool is too small).
 */
int apm_streamer_set_host_first_page(apm_streamer* s, int64_t first_model_page);

/* Restricts the step calls of `s` to model pages [0, n_pages) (n_pages < 0: all pages in use); the
 * pages beyond are some other handle's (apm_tiered_set_range).  Not with the scheduled step. */
int apm_streamer_set_page_count(apm_streamer* s, int64_t n_pages);

/*
 * Measurement aid (staged modes only): the same pipeline (streams, events, copy sizes, slot reuse)
 * with the kernels left out.  directions: 1 = copy-in only, 2 = copy-out only, 3 = both.  The data make a round
 * trip host -> staging -> host, so the host pool's contents are unchanged (with 2 alone, staging
 * contents left by an earlier step are written back: call it only after 1 or 3, or a full step).
 */
int apm_streamer_copy_only(apm_streamer* s, int directions, void* stream);

/* ---- life-time based scheduling of page movement (Alg. 1, phase 1) ------------------------- */

/*
 * A task of the schedule (Alg. 1's {operation, page, trigger_id}): target is a page id for
 * APM_TASK_MOVE_TO_GPU and a layer index for APM_TASK_COMPUTE; trigger_id is the logical id (layer
 * index) at which the task is issued.  Tasks run in list order; a movement task that follows a
 * compute task in the list may use memory that compute released.
 */
enum apm_task_op { APM_TASK_MOVE_TO_GPU = 0, APM_TASK_COMPUTE = 1 };
typedef struct apm_task {
    int32_t op;
    int32_t trigger_id;
    int64_t target;
} apm_task;

/*
 * Host-only planner.  The model is n_layers layers in execution order; layer i first accesses the
 * pages layer_pages[layer_offsets[i] .. layer_offsets[i+1]) (every page id in [0, n_pages) in
 * exactly one layer) and needs layer_bytes[i] bytes besides its pages while it computes.  The trace
 * is last_access[page] = index of the layer that accesses the page last, after whose compute the
 * page's GPU memory is free again (NULL: the page's own layer).
 * Phase 1 of Alg. 1: all movement tasks are put first; per layer, movement tasks are taken off the
 * end of the schedule while less than layer_bytes[i] would be left, the compute is appended, and
 * deferred pages are put back, earliest needed first, while more than one page of memory is left.
 * Readings where the listing is silent: a page of layer i still deferred when i's turn comes is
 * moved then (trigger i); a layer that cannot fit even with all later pages deferred is an error.
 * Phase 2 re-times all_gather tasks only and has nothing to do on one GPU.
 *
 * All pointers are host pointers.  tasks: capacity *n_tasks on entry, count (n_pages + n_layers)
 * on return (NULL with *n_tasks == 0 queries the count); peak_bytes (nullable): the largest
 * resident pages + layer_bytes over all computes.
 * Errors: APM_EINVAL (malformed arrays, a page in two layers, last_access before the page's own
 * layer), APM_ERANGE (page id out of range; task buffer too small), APM_ENOMEM (some layer does
 * not fit into gpu_memory_bytes; the message names it).
 */
int apm_schedule_plan(const int64_t* layer_offsets, const int64_t* layer_pages,
                      const int64_t* layer_bytes, int64_t n_layers, const int64_t* last_access,
                      int64_t n_pages, int64_t page_bytes, int64_t gpu_memory_bytes,
                      apm_task* tasks, int64_t* n_tasks, int64_t* peak_bytes);

/*
 * One AdamW step over all pages in use, with the page movement driven by a schedule (the task
 * list of apm_schedule_plan, or any list that passes the checks below) instead of the staged
 * mode's fixed slot ring.  The model's layers are consecutive page ranges: layer i owns pages
 * [layer_first_page[i], layer_first_page[i+1]) (n_layers + 1 host entries, from 0 to the number of
 * pages in use) and updates them when it computes.  last_access (host pointer, one entry per page
 * in use, nullable = each page's own layer) is the trace the schedule was planned with: a page
 * stays in GPU memory until the layer last_access[page] >= its own layer has computed.  The GPU
 * memory of the schedule is the streamer's staging memory: n_slots * batch_pages page slots of
 * 12 * page_elems bytes (p, m, v).  APM_TASK_MOVE_TO_GPU copies a page's fp32 classes from the
 * host pool into the lowest free slot; APM_TASK_COMPUTE runs the reduce and update kernels on its
 * layer's pages, then copies the pages whose last access it is back to the host pool and frees
 * their slots.  Movement tasks over consecutive pages and slots with one trigger id are merged
 * into one copy per class.
 * Dispatch is event-driven (Sec. 5 "Unified Scheduler"): a movement task is never issued before
 * execution has reached its trigger_id -- the layer before it has computed (trigger 0: the start
 * of the step) -- nor before the slots it moves into have been written back; a compute starts
 * when the movements of its pages have completed; a write-back when its compute has.  A movement
 * may be issued later than its trigger allows: with the library's copy kernel as the mover, a
 * movement that is due waits for the next write-back and crosses the link in the same kernel (the
 * two directions in one kernel are a fifth faster than in two), at the latest two units ahead of
 * the compute that needs its page, or right before that compute if it was not due earlier; and a
 * compute task is then carried out in units of at most 16 pages, each written back as soon as it
 * has computed (the pages of the optimizer pass are independent), so a slot may become free
 * earlier than the schedule says, never later.
 * The schedule is replayed on the host first and nothing is enqueued if it is unsound:
 * APM_ENOMEM (a movement task finds no free slot), APM_ESTATE (a layer computes before all its
 * pages were moved; a resident cache is set), APM_EINVAL (layers out of order, a page moved twice,
 * pages or layers left over, a trigger id beyond the layers that precede the task in the list,
 * last_access before a page's own layer).  Results are bit-identical to the other modes.  Stream
 * semantics as apm_streamer_step.  Pages move by the library's copy kernel (used extents only),
 * or by the runtime's copies, each movement issued at its trigger, if the streamer is in
 * APM_STREAM_STAGED_DMA mode or the GPU cannot address the host pool.
 */
int apm_streamer_step_scheduled(apm_streamer* s, const apm_task* tasks, int64_t n_tasks,
                                const int64_t* layer_first_page, int64_t n_layers,
                                const int64_t* last_access, int64_t step, const apm_hyper* hyper,
                                float* grad_norm, uint8_t* skip_mask, void* stream);

/* ---- third tier: FP32 states in files (the device map's SSD, Sec. 4.1; Alg. 2 fetches the
 *      states from SSD, updates them and offloads them back) ---------------------------------- */

/*
 * A pool whose state classes live in files <path_prefix>.p32 / .m32 / .v32 / .g16 / .p16 (one per
 * class in state_mask), each n_pages * page_elems elements, page k at byte offset k * page bytes.
 * Without APM_POOL_NO_ZERO the files are created anew and read as zeros; with it, existing files
 * are opened as they are (and extended with zeros to full size).  APM_POOL_FILE_DIRECT needs
 * pages of a multiple of 4096 bytes.  The files are not removed by apm_pool_destroy.
 * A FILE pool has no layout of its own and exchanges pages with HOST pools only:
 * apm_page_copy_async between a FILE and a HOST pool synchronises `stream`, then reads or writes
 * the pages before it returns (file I/O is not stream-ordered).  No GPU is needed to create one.
 * Errors: APM_EINVAL, APM_EDEVICE (the file cannot be created; the message has the reason).
 */
int apm_file_pool_create(apm_pool** out, const char* path_prefix, int32_t hip_device,
                         int64_t page_elems, int64_t n_pages, uint32_t state_mask, uint32_t flags);

/*
 * Streamed update over file-resident state.  file: FILE pool storing P32, M32, V32; dev: GPU pool
 * storing G16 and P16 with an installed layout (same page size).  The only staging is a window of
 * pinned host memory, n_slots slots of batch_pages pages x 3 classes: io_threads I/O threads read
 * the next batches into free slots and write finished ones back, in pieces of 8 MiB, while the
 * update kernel works on the current batch directly in the window across PCIe (as in
 * APM_STREAM_DIRECT).  n_slots >= 2, io_threads in [1, 64].
 */
int apm_tiered_create(apm_tiered** out, apm_pool* file, apm_pool* dev, int64_t batch_pages,
                      int n_slots, int io_threads);
int apm_tiered_destroy(apm_tiered* t); /* before the pools it uses */

/*
 * Restricts the step calls of `t` to model pages [first_page, first_page + n_pages) (n_pages < 0:
 * to the last page in use); file page k is model page k as before.  With
 * apm_streamer_set_page_count this composes the paper's three levels on one GPU pool (Sec. 4.2,
 * Sec. 4.3): the leading pages cached in HBM, the next in pinned host memory (both one
 * apm_streamer_step), the rest in files (one apm_tiered_step).  Per-page outputs stay indexed by
 * model page.  Only one of the handles on a GPU pool may drive the one-step-stale form.
 */
int apm_tiered_set_range(apm_tiered* t, int64_t first_page, int64_t n_pages);

/* Measurement aid: bytes queued for reading from / writing to the files since creation (host
 * pointers, nullable). */
int apm_tiered_io_bytes(apm_tiered* t, int64_t* bytes_read, int64_t* bytes_written);

/*
 * One AdamW step over all pages in use.  The kernels start after everything enqueued on `stream`
 * so far; the call blocks the calling thread until the last page has been written back (so,
 * unlike the other step calls, it is synchronous).  grad_norm / skip_mask as in
 * apm_page_adamw_step.  Results are bit-identical to the resident update.
 * With APM_SKIP_UNTOUCHED, the pages that are skipped (decided by one reduce pass over all
 * gradients, which live in HBM) are neither read from nor written to the files: I/O is
 * proportional to the pages that receive a gradient (the experts a step routed tokens to).
 * Errors: as apm_page_adamw_step, and APM_EDEVICE if a read or write fails (the step still drains;
 * the files may then hold a partly updated state).
 */
int apm_tiered_step(apm_tiered* t, int64_t step, const apm_hyper* hyper, float* grad_norm,
                    uint8_t* skip_mask, void* stream);

/*
 * Alg. 2 with its two actors as two host threads.  The call (1) waits for the update started by
 * the previous call, (2) if a gradient is buffered, counts it as applied and starts the library's
 * updater thread on it (the step above, reading the buffered gradient, once its staging has
 * completed), (3) stages new_g16 (device pointer, page layout, all pages in use) into the other
 * half of the GPU pool's ping-pong buffer on `stream` and returns; the caller produces the next
 * gradient while the updater fetches, updates and offloads the states.  new_g16 == NULL flushes:
 * the buffered gradient is applied and the call returns when that update is complete.
 * N calls + flush leave exactly the state of N apm_tiered_step calls with the same per-call
 * hyper-parameters: a gradient is applied with the values of the call that brought it (copied
 * then), not of the call that starts its update.  While an update runs, the
 * GPU pool's per-page scratch is in use: no other step call on that pool (apm_delayed_accumulate
 * into the gradient being collected is fine: Alg. 2's buffering actor).  The applied counter
 * and apm_delayed_set_outputs are those of the GPU pool; apm_delayed_grad_buffer is not available
 * here (APM_EINVAL).  An error of the background update is reported by the next call.
 */
int apm_tiered_step_delayed(apm_tiered* t, const void* new_g16, const apm_hyper* hyper, void* stream);

/* ---- one-step-stale update (Alg. 2 reduced to one GPU: apply the buffered gradient while the
 *      next one is being staged) -------------------------------------------------------------- */

/*
 * new_g16 != NULL: device pointer to a gradient for the whole pool in page layout (capacity
 * n_pool_pages*E bf16 elements; only the used extents of the listed pages are read).  The call
 *   (1) if a gradient is buffered, increments the pool's applied-update counter c and enqueues the
 *       AdamW step with t = c on the buffered gradient on the pool's internal update stream;
 *   (2) enqueues, on `stream`, the staging of new_g16 into the other half of the pool's ping-pong
 *       gradient buffer; the caller may reuse new_g16 once `stream` has passed this point.
 * new_g16 == NULL flushes: applies the buffered gradient if any and makes `stream` wait for the
 * update stream.
 * A gradient is buffered together with the page list (as in apm_page_adamw_step; copied) and the
 * hyper-parameters (copied) of the call that brings it, and is applied with those one call later:
 * under a learning-rate schedule gradient t meets lr_t although call t+1 enqueues its update, so N
 * calls and a flush leave exactly the state of N apm_page_adamw_step calls with the same
 * per-call arguments.  The hyper-parameters passed with a flush are validated and otherwise unused.
 * P16 is rewritten asynchronously by the update stream: a reader that does not flush may see
 * parameters one step stale, which is the mechanism's stated trade-off.
 */
int apm_step_delayed(apm_pool* pool, const int64_t* pages, int64_t n_pages, const void* new_g16,
                     const apm_hyper* hyper, void* stream);

/*
 * The same hand-over with the fp32 state in host memory (Alg. 2's setting: the updating side works
 * on states that do not live on the GPU): what is applied is one apm_streamer_step over all pages
 * in use, on the GPU pool's update stream, reading the buffered gradient; what is staged is
 * new_g16 (page layout, as above; NULL flushes).  In direct mode the update occupies 64
 * wavefronts, so the producer's kernels on `stream` keep the rest of the GPU.  The ping-pong
 * halves, the applied counter, apm_delayed_grad_buffer, apm_delayed_accumulate and
 * apm_delayed_set_outputs are those of the streamer's GPU pool.  As with apm_step_delayed, a
 * gradient is applied with the hyper-parameters of the call that brought it.
 */
int apm_streamer_step_delayed(apm_streamer* s, const void* new_g16, const apm_hyper* hyper,
                              void* stream);

/*
 * Whether the one-step-stale form can overlap at all: the runtime maps streams onto a few hardware
 * queues, and kernels of two streams that share a queue run one after the other.  On the first
 * apm_step_delayed / apm_streamer_step_delayed call with a given producer stream (and after a mode
 * change) the library therefore measures, with two spin kernels of half a millisecond, whether
 * its update stream and the streamer's pipeline streams run beside `stream`, and replaces those
 * that do not by streams that do; this synchronises the device once.  The report: 1 = runs beside
 * the producer stream, 0 = no such stream was found (the update then runs after the producer's
 * work, never wrongly), -1 = not measured yet.  Host pointers, nullable.
 */
int apm_streamer_overlap_report(const apm_streamer* s, int* update_stream, int* pipeline_streams);

/*
 * Adds one more gradient into the gradient buffered by the last apm_step_delayed call, before the
 * next call applies it (Alg. 2, buffering thread: g'16 <- g'16 + g16): element-wise
 * bf16_rne(fp32(g') + fp32(g)), the fp32 sum rounded to nearest, over the used extents of the
 * listed pages.  g16: device pointer, page layout, as new_g16 of apm_step_delayed.  Asynchronous
 * on `stream`; the caller may reuse g16 once `stream` has passed this point.
 * Errors: APM_ESTATE if no gradient is buffered; APM_EINVAL, APM_ERANGE.
 */
int apm_delayed_accumulate(apm_pool* pool, const int64_t* pages, int64_t n_pages, const void* g16,
                           void* stream);

/*
 * Zero-copy hand-over for apm_step_delayed: returns the half of the ping-pong gradient buffer the
 * next call will stage into (device pointer, n_pool_pages*E bf16 elements in page layout) and
 * makes `stream` wait until the update that last read that half has finished.  A producer that
 * writes its gradient there (on `stream`) and passes the same pointer as new_g16 skips the
 * staging copy.  Both halves start zero-filled; the producer must leave the elements no tensor
 * owns (alignment gaps, padding) zero.  The pointer is valid for exactly one apm_step_delayed
 * call.  NULL on error.
 */
void* apm_delayed_grad_buffer(apm_pool* pool, void* stream);

/* Number of updates apm_step_delayed has applied (enqueued) on this pool so far. */
int64_t apm_delayed_applied(const apm_pool* pool);

/* Per-page outputs of the delayed path: device pointers (float[n] / uint8_t[n], nullable) the
 * update kernels of later apm_step_delayed calls write, indexed like their page list. */
int apm_delayed_set_outputs(apm_pool* pool, float* grad_norm, uint8_t* skip_mask);

#ifdef __cplusplus
}
#endif
#endif /* APM_H */
