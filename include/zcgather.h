/*
 * zcgather -- GPU-issued sparse row gather from pinned, device-mapped host
 * memory into a dense tensor in HBM, for one MI355X (gfx950).
 *
 * The method (paper Sections 3.1-3.3): the node-feature table stays in host
 * memory that is page-locked and mapped into the GPU address space; for each
 * minibatch the GPU itself reads the rows named by the sampled node-ID list
 * over the host link ("zero-copy") and writes them densely into GPU memory,
 * instead of a CPU gather into a staging buffer followed by a DMA copy.
 *
 * Conventions
 *  - C ABI, no exceptions; every call returns an int status: ZCG_OK (0) or a
 *    negative ZCG_E* code. zcg_strerror() names a code; when the code is
 *    ZCG_EHIP, zcg_last_hip_error() gives the HIP error of the calling thread.
 *  - "host" pointers are ordinary process addresses; "device" pointers are
 *    addresses valid in GPU kernels (HBM or mapped host memory).
 *  - Tables are row-major, contiguous: row r occupies bytes
 *    [r*row_bytes, (r+1)*row_bytes), row_bytes = dim * element size.
 *  - Handles may be used from several threads; creating and destroying
 *    handles is serialised inside the library.
 */
#ifndef ZCGATHER_H
#define ZCGATHER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------ */
#define ZCG_OK 0
#define ZCG_EINVAL (-1)  /* null pointer, non-positive size, bad option value   */
#define ZCG_EDTYPE (-2)  /* dtype is not one of the ZCG_* element types          */
#define ZCG_EHANDLE (-3) /* not a live table handle (never made, or destroyed)  */
#define ZCG_EHIP (-4)    /* a HIP runtime call failed; see zcg_last_hip_error() */
#define ZCG_ENOMEM (-5)  /* host allocation failed                              */
#define ZCG_EALIGN (-6)  /* pointer not aligned to the element size             */
#define ZCG_EALIAS (-7)  /* ranges that must be distinct overlap (output/table ...) */
#define ZCG_ERANGE (-8)  /* an index is outside [0, n_rows) (host-side checks)  */
#define ZCG_EBUSY (-9)   /* pipeline: the next buffer has not been released yet */
#define ZCG_ETIMEDOUT (-10) /* pipeline: a bounded wait ran out                   */
#define ZCG_ECLOSED (-11)   /* pipeline: the producer has finished                */
#define ZCG_ECAPACITY (-12) /* input larger than a fixed capacity of the entry point */

/* ---- element types: only the size matters, payload bits are never read -- */
#define ZCG_F16 1 /* 2-byte elements (fp16, bf16, int16)         */
#define ZCG_F32 2 /* 4-byte elements (fp32, int32)               */
#define ZCG_B8 3  /* 1-byte elements (int8, fp8 feature tables)  */
#define ZCG_B64 4 /* 8-byte elements (fp64, int64)               */

/* ---- allocation flags for zcg_alloc_table ------------------------------ */
#define ZCG_ALLOC_DEFAULT 0u     /* pinned, mapped, coherent (fine-grained)         */
#define ZCG_ALLOC_NONCOHERENT 1u /* pinned, mapped, non-coherent: the GPU may cache
                                    lines; host writes made while a kernel runs are
                                    not guaranteed visible to it                      */
#define ZCG_ALLOC_NUMA_USER 2u   /* keep the calling thread's NUMA policy           */
#define ZCG_ALLOC_UNCACHED 4u    /* pinned, mapped, extended fine-grained pool: the
                                    GPU does not cache the table at all               */

/* ---- gather kernels (zcg_gather_variant / zcg_gather_ex) --------------- */
#define ZCG_VARIANT_AUTO 0    /* rows shorter than a line or made of whole lines: ROWVEC;
                                 else ALIGNED, or HALFLINE for host-resident rows of more
                                 than a line (also for multi-pass whole-line rows off
                                 the 256-byte pair grid). With workspace lent through
                                 zcg_launch_opts, long dense lists of host-resident rows
                                 of at most a line are walked in ascending table order.  */
#define ZCG_VARIANT_NAIVE 1   /* one element per lane over the flat output, no alignment
                                 care: the paper's baseline kernel (Section 4.1.2 (c))  */
#define ZCG_VARIANT_ROWVEC 2  /* a lane group per row, widest vector, loads start at the
                                 row start                                              */
#define ZCG_VARIANT_ALIGNED 3 /* a lane group per row; loads start at the line boundary
                                 below the row start and are masked to the row, so every
                                 wave load covers whole lines: the goal of the paper's
                                 circular shift (Section 3.2.1), reads aligned, the
                                 misalignment moved to the local writes                */
#define ZCG_VARIANT_HALFLINE 4 /* ALIGNED, and row ends that occupy at most half a line are
                                  fetched as 64-byte reads through the scalar data cache:
                                  on gfx950 a vector load of host memory always costs the
                                  whole 128-byte line on the link, a scalar load half of
                                  it. Needs loads of 4 bytes or more (vec_bytes >= 8 with
                                  shifted stores when rows or bases are only 1- or 2-byte
                                  granular), else ALIGNED.                              */
#define ZCG_VARIANT_COUNT 5

typedef struct zcg_table zcg_table; /* opaque */

/* Launch options for zcg_gather_ex. Zero in any field means "library default". */
typedef struct zcg_launch_opts {
  int variant;     /* ZCG_VARIANT_*                                                   */
  int max_blocks;  /* cap on the grid size (blocks of 256 lanes); the kernels stride   */
  int unroll;      /* independent loads in flight per lane: 1, 2, 4 or 8               */
  int line_bytes;  /* alignment target of ALIGNED: 32, 64, 128 or 256 (default 128; 256
                      for host-resident rows that take several wave passes)            */
  int nt_loads;    /* 1: non-temporal table loads, 2: plain loads, 3: system scope;
                      default: plain for host tables, non-temporal for HBM tables      */
  int nt_stores;   /* 1: non-temporal output stores, 2: plain stores                   */
  int vec_bytes;   /* cap on bytes per lane access: 1, 2, 4, 8 or 16 (>= element size)  */
  int group_lanes; /* lanes given to one row, a power of two up to 64; raised to what
                      the row needs. 64 = one row per wave-wide load instruction       */
  int shifted_stores; /* ALIGNED / HALFLINE with rows or bases less aligned than vec_bytes: 1 (and the
                      default) keeps the loads vec_bytes wide at line-aligned positions and
                      writes with narrower / unaligned stores; 2 narrows the loads instead.
                      With wide loads, up to vec_bytes-1 bytes next to a row end, inside
                      the same aligned vec_bytes block, are read and dropped.            */
  int row_splits;  /* rows wider than one wave pass: number of wavefronts that share a
                      row, each taking one contiguous piece (1 = one wavefront per row,
                      up to 4096). Default: 1 for long lists; short lists of long rows
                      are split until there is enough work in flight to fill the link.
                      HALFLINE and NAIVE do not split.                                  */
  int half_ends;   /* HALFLINE: 1 = every row end that fits half a line goes through a
                      64-byte scalar read; 2 = only ends whose line would otherwise be
                      requested alone (its partner in the 256-byte aligned pair is not
                      part of the row), which never adds a link request. Default: 1 for
                      rows of 768 bytes and more, 2 for shorter rows.                   */
  void* workspace_dev;     /* optional: device memory, CALLER-OWNED, 256-byte aligned, that
                      the call may overwrite while it runs on its stream (free to reuse
                      once the stream has passed the call; two calls that overlap in
                      time need two workspaces). With variant AUTO and at least
                      zcg_gather_workspace_bytes(n_idx) bytes, zcg_gather_ex walks lists
                      of host-resident rows of at most 128 bytes in ascending table
                      order where that pays: it builds the order in the workspace with
                      a few kernels of its own on the same stream (0.04-0.09 ms), then
                      gathers through it. The result is the same bit for bit; listed
                      rows that share a line or a 256-byte pair of lines then share a
                      link request, so the walk pays for long lists that are dense in
                      their table (decided from n_idx, n_rows and the row size).
                      Ignored otherwise, and by every forced variant. When it is used it
                      must not overlap the list, the table or the output (ZCG_EALIAS).  */
  int64_t workspace_bytes; /* size of workspace_dev in bytes (0 with a null pointer)       */
} zcg_launch_opts;

/* How one gather call is laid out on the GPU; filled by zcg_plan_gather. */
typedef struct zcg_plan {
  int variant;     /* resolved: NAIVE, ROWVEC, ALIGNED or HALFLINE                     */
  int vec_bytes;   /* bytes per lane access                                            */
  int log2_group;  /* lanes per row = 1 << log2_group (row kernels)                    */
  int iters;       /* group-wide passes needed to cover the widest (aligned) row span  */
  int unroll;      /* independent loads in flight per lane                             */
  int line_bytes;  /* alignment target (ALIGNED)                                       */
  int nt_loads;    /* 0 plain, 1 non-temporal, 2 system scope                          */
  int nt_stores;   /* 0 / 1                                                            */
  int blocks;      /* grid size, blocks of 256 lanes                                   */
  int store_bytes; /* alignment the stores can rely on; < vec_bytes means shifted stores */
  int row_splits;  /* wavefronts per row (rows wider than one wave pass), else 1          */
  int half_ends;   /* HALFLINE: 1 all row ends, 2 lone lines only; else 0                 */
  int ordered;     /* 1: zcg_gather_ex with these options would build the ascending order in
                      the lent workspace and walk the list through it; else 0             */
} zcg_plan;

/* ---- errors ------------------------------------------------------------ */
const char* zcg_strerror(int status);
int zcg_last_hip_error(void); /* hipError_t of the last failed HIP call on this thread */

/*
 * Step "map the table" (Section 3.1: page-lock an existing host buffer and map
 * it into the GPU address space; no data is copied).
 * host_ptr: host, CALLER-OWNED, n_rows*dim*elem bytes, must stay valid and
 * unmoved until zcg_unregister_table. Pins with hipHostRegister (mapped,
 * portable) on `device`. Errors: ZCG_EINVAL (null, n_rows<=0, dim<=0),
 * ZCG_EDTYPE, ZCG_EALIGN, ZCG_EHIP (pin or map refused; nothing stays pinned).
 * Some installations refuse hipHostRegister for memory that already exists (the
 * machines this library was measured on do: there this call returns ZCG_EHIP and
 * has only had its argument checks exercised); zcg_alloc_table always works, and
 * zcg_table_view gives tables that start anywhere inside such an allocation.
 */
int zcg_register_table(void* host_ptr, int64_t n_rows, int64_t dim, int dtype, int device,
                       zcg_table** out);

/*
 * Same step with LIBRARY-OWNED memory: hipHostMalloc (mapped, portable, plus
 * `flags`). The caller fills the table through zcg_table_host_ptr(). Contents
 * are uninitialised. Freed by zcg_unregister_table.
 */
int zcg_alloc_table(int64_t n_rows, int64_t dim, int dtype, unsigned flags, int device,
                    zcg_table** out);

/*
 * Wrap a table that already lives in GPU memory (the paper's "all-in-GPU"
 * comparison, Section 4.1.2 (d)): dev_ptr is device, CALLER-OWNED.
 */
int zcg_table_from_device(void* dev_ptr, int64_t n_rows, int64_t dim, int dtype, int device,
                          zcg_table** out);

/*
 * A slice of a live table as a table of its own: rows of `dim` elements of
 * `dtype` starting `byte_offset` bytes into the parent's memory (Section 3.1: the
 * unified tensor is made from an EXISTING buffer, whose address and alignment the
 * library does not choose -- a sub-tensor of a larger pinned allocation, a table
 * with a header in front of it). No memory is pinned or copied; the view reads
 * through the parent's mapping and stays host-resident if the parent is. It must
 * lie inside the parent (ZCG_EINVAL), start on an element boundary (ZCG_EALIGN),
 * and is dead once the parent is unregistered (ZCG_EHANDLE from then on);
 * unregister the view itself to free its handle.
 */
int zcg_table_view(const zcg_table* parent, int64_t byte_offset, int64_t n_rows, int64_t dim,
                   int dtype, zcg_table** out);

/* Accessors; return NULL / 0 for a handle that is not live. */
void* zcg_table_device_ptr(const zcg_table* t); /* pointer kernels read the table through */
void* zcg_table_host_ptr(const zcg_table* t);   /* host address, NULL for device tables    */
int64_t zcg_table_row_bytes(const zcg_table* t);
int64_t zcg_table_n_rows(const zcg_table* t);

/*
 * Unpin / free. The handle is dead afterwards; a second call, or a pointer that
 * was never a handle, returns ZCG_EHANDLE. The caller must first make sure no
 * gather that reads the table is still running.
 */
int zcg_unregister_table(zcg_table* t);

/*
 * The gather (Section 3.2.1, Listing 2 semantics; Section 3.3: the index list
 * is already on the GPU, the result lands in a GPU buffer):
 *     out[i, c] = table[idx[i], c],  0 <= i < n_idx, 0 <= c < dim,
 * bit for bit. Asynchronous: enqueues one kernel on `stream` (a hipStream_t
 * passed as void*; NULL = the default stream) and returns; no allocation, no
 * synchronisation, no host read of idx_dev.
 *   idx_dev : device, n_idx int64, each in [0, n_rows). Out-of-range entries
 *             are NOT checked here (undefined behaviour, as in the paper's
 *             kernel); use zcg_validate_indices when in doubt. Any address the
 *             GPU can read will do, mapped pinned host memory included (the
 *             list is then fetched over the link too, 8 bytes per row).
 *   out_dev : device, CALLER-OWNED, n_idx*row_bytes bytes, aligned to the
 *             element size (16-byte alignment enables the widest accesses),
 *             must not overlap the table, the list or a caller's order
 *             (ZCG_EALIAS).
 * The caller keeps idx_dev, out_dev and the table alive until the stream has
 * passed the kernel. n_idx == 0 succeeds without a launch. The table must not
 * change while a gather that reads it runs; rows the host rewrites after a
 * gather has completed are seen by every later gather (the GPU's caches, the
 * scalar cache included, are invalidated when a kernel starts).
 * Safe under stream capture (one kernel node, nothing else is recorded): a
 * replayed graph reads whatever idx_dev and the table hold at replay time.
 * Calls on one handle may come from any number of host threads and streams.
 */
int zcg_gather(const zcg_table* t, const int64_t* idx_dev, int64_t n_idx, void* out_dev,
               void* stream);

/* Same, forcing one kernel (ablation: Section 4.2 compares naive and aligned). */
int zcg_gather_variant(const zcg_table* t, const int64_t* idx_dev, int64_t n_idx, void* out_dev,
                       void* stream, int variant);

/* Same, with every launch knob exposed (opts may be NULL). */
int zcg_gather_ex(const zcg_table* t, const int64_t* idx_dev, int64_t n_idx, void* out_dev,
                  void* stream, const zcg_launch_opts* opts);

/*
 * The same gather with a processing order: work item k fetches row idx[order[k]]
 * and writes output row order[k], so the result is exactly zcg_gather's, but the
 * table is walked in the order given. With order = the permutation that sorts
 * idx ascending (zcg_make_order), neighbouring work items touch neighbouring
 * lines and pages of the host table: repeated and adjacent rows share link
 * requests. Pays on short rows (measured +35 % on 32-byte rows, +12 % on
 * 128-byte rows, sort included it still wins below ~128 bytes per row).
 *   order_dev : device, n_idx int64, a permutation of [0, n_idx); entries outside
 *               that range are undefined behaviour
 * NAIVE has no ordered form (ZCG_EINVAL).
 */
int zcg_gather_ordered(const zcg_table* t, const int64_t* idx_dev, const int64_t* order_dev,
                       int64_t n_idx, void* out_dev, void* stream, const zcg_launch_opts* opts);

/*
 * Builds that order on the GPU: a stable least-significant-digit radix sort of
 * (idx[i], i) by idx, hand-written for wave64 (digits of up to 8 bits; per digit a
 * count, a prefix and a scatter kernel; deterministic). Equal indices keep their
 * list order. Asynchronous on `stream`; allocates nothing: all temporary memory is
 * the caller's workspace (device, 256-byte aligned, at least
 * zcg_order_workspace_bytes(n_idx) bytes = about 9 bytes per entry,
 * free to reuse once the stream has passed the call). order_dev itself is used as
 * a second buffer while the order is built. n_rows bounds the index values: only
 * the bits below it are sorted, so entries outside [0, n_rows) still yield a
 * permutation, just not an ascending one. n_idx < 2^32 (ZCG_EINVAL beyond). The
 * list, the order and the workspace must not overlap (ZCG_EALIAS).
 * Safe under stream capture: only kernel nodes are recorded.
 */
int zcg_order_workspace_bytes(int64_t n_idx, int64_t* bytes);
int zcg_make_order(const int64_t* idx_dev, int64_t n_idx, int64_t n_rows, int64_t* order_dev,
                   void* workspace_dev, int64_t workspace_bytes, void* stream);

/*
 * zcg_make_order for callers that cannot allocate or lend device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same order, same kernels; the temporary memory is a static device array inside
 * the library (9.1 MiB on every GPU the library runs on, held until the process
 * ends) instead of a workspace argument. The call allocates nothing.
 *   n_idx <= ZCG_STATIC_ORDER_MAX_IDX (ZCG_ECAPACITY beyond: use zcg_make_order with
 *   a workspace); other arguments and errors as zcg_make_order. Works on the
 *   current device.
 * Every call on one GPU shares that GPU's array: two calls that overlap in time
 * on one GPU (different streams, no ordering between them) race and give a wrong
 * order; calls on one stream, or ordered by events, are fine. Nothing in the array
 * has to be cleared between calls. The first call on a device looks the array's
 * address up once; make that call outside stream capture.
 */
#define ZCG_STATIC_ORDER_MAX_IDX 1048576
int zcg_make_order_static(const int64_t* idx_dev, int64_t n_idx, int64_t n_rows, int64_t* order_dev,
                          void* stream);

/* Bytes of zcg_launch_opts.workspace_dev that let zcg_gather_ex order a list of n_idx
 * entries by itself: the order (8 bytes per entry) plus zcg_order_workspace_bytes. */
int zcg_gather_workspace_bytes(int64_t n_idx, int64_t* bytes);

/*
 * Host-only: the launch shape zcg_gather_ex would use for this table, output
 * address and options (no GPU call is made). For tests and for reasoning about
 * which bytes each wave load covers.
 */
int zcg_plan_gather(const zcg_table* t, int64_t n_idx, const void* out_dev,
                    const zcg_launch_opts* opts, zcg_plan* plan);

/*
 * The same planning for a table described by numbers instead of a handle: rows of row_bytes
 * bytes made of elem_bytes-byte elements (1, 2, 4 or 8) starting at table_addr, output at
 * out_addr, host_resident != 0 for a table read over the host link. Host-only, no GPU needed:
 * lets a caller (or a test) see which kernel and launch shape any address, row size and option
 * set would get. `ordered` in the result tells whether a lent workspace would be used, judged
 * with n_rows rows in the table. Errors as zcg_gather_ex's argument checks.
 */
int zcg_plan_shape(int64_t row_bytes, int elem_bytes, uint64_t table_addr, uint64_t out_addr,
                   int64_t n_rows, int64_t n_idx, int host_resident, const zcg_launch_opts* opts,
                   zcg_plan* plan);

/*
 * Debug helper, SYNCHRONOUS: counts entries of idx_dev outside [0, n_rows) on
 * the GPU, waits, and writes the count to *n_bad_host (host). Allocates and
 * frees 8 bytes of device memory.
 */
int zcg_validate_indices(const zcg_table* t, const int64_t* idx_dev, int64_t n_idx, void* stream,
                         int64_t* n_bad_host);

/*
 * The DMA-based method the paper argues against (Section 4.1.2 (b)): CPU
 * threads gather the rows into a dense staging buffer, then ONE host-to-device
 * copy moves it. Reported as a baseline.
 *   idx_host       : host, n_idx int64; checked while gathering, ZCG_ERANGE on a bad entry
 *                    (out_dev then holds nothing of this call; the chunked form may
 *                    already have copied the chunks before the bad entry)
 *   staging_pinned : host, CALLER-OWNED, >= n_idx*row_bytes bytes, should be
 *                    pinned (hipHostMalloc) for the copy to be asynchronous
 *   n_threads      : CPU threads for the gather (<=0: all available)
 * The gather runs before the call returns; the copy is enqueued on `stream`
 * and may still be in flight. Only for host-resident tables (ZCG_EINVAL else).
 */
int zcg_cpu_gather_memcpy(const zcg_table* t, const int64_t* idx_host, int64_t n_idx,
                          void* staging_pinned, void* out_dev, int n_threads, void* stream);

/*
 * Strongest form of the same baseline: the list is cut into chunks of
 * `chunk_rows` rows; the CPU gathers chunk k+1 while the copy of chunk k is in
 * flight. staging_pinned must hold the whole gathered result.
 */
int zcg_cpu_gather_memcpy_chunked(const zcg_table* t, const int64_t* idx_host, int64_t n_idx,
                                  void* staging_pinned, void* out_dev, int n_threads,
                                  int64_t chunk_rows, void* stream);

/*
 * Resource provisioning (Section 3.2.2: the gather needs only a small share of
 * the GPU to saturate the link, the rest stays free for compute kernels). The
 * paper caps the gather's share with a process-level service; here a stream is
 * bound to a set of compute units instead, inside one process.
 *   mask_words : host, n_words x 32 bits, bit i = compute unit i may run work of
 *                this stream; at least one bit must be set among the device's CUs
 * On this chip bit i is compute unit i/8 of accelerator die i%8, and the runtime
 * refuses (ZCG_EHIP) a mask that leaves one of the 8 dies without a compute
 * unit: the first n bits with n a multiple of 8 give n/8 units on every die.
 * Default priority. Destroy with zcg_stream_destroy (waits for the stream).
 */
int zcg_stream_create_cu_mask(int device, const uint32_t* mask_words, int n_words, void** stream);
int zcg_stream_destroy(void* stream);
int zcg_device_cu_count(int device, int* n_cus);

/*
 * Minibatch pipeline, producer side (Section 3.3: sampler -> producer -> consumer
 * with alternating GPU buffers and one synchronisation per minibatch). One
 * process; the producer's gather stream and the caller's consumer stream meet
 * through events.
 *   out_bufs      : host array of n_buffers (1..16) device pointers, CALLER-OWNED,
 *                   each >= max_rows*row_bytes bytes; the ring of output buffers
 *   gather_stream : stream the list copies and gathers run on (e.g. one from
 *                   zcg_stream_create_cu_mask); NULL = the pipeline creates its own
 * The pipeline owns, per buffer, a pinned staging area and a device copy of the
 * index list (max_rows int64 each). For tables of at most 2^32 rows the list is
 * staged as 32-bit values that a small kernel on the gather stream reads straight
 * from the staging area and widens (half the bytes over the link, no copy engine). For host-resident tables with rows of at
 * most 128 bytes it also owns the memory of zcg_make_order and gathers lists
 * that are long and dense enough in the table in ascending table order (same
 * result, fewer link requests). Threads: ONE producer thread (submit,
 * submit_wait, finish) and ONE consumer thread (next, acquire, release) may run
 * at the same time; they may also be the same thread. The consumer takes slot
 * numbers either from submit's result or from zcg_pipeline_next, not from both.
 */
typedef struct zcg_pipeline zcg_pipeline;
int zcg_pipeline_create(const zcg_table* t, int64_t max_rows, int n_buffers, void* const* out_bufs,
                        void* gather_stream, zcg_pipeline** out);
/*
 * Producer: stage the list (host, checked: ZCG_ERANGE), bring it to the GPU and enqueue
 * the gather into the next buffer of the ring, behind the consumer's release of
 * that buffer. Returns at once unless the producer is a whole ring ahead of its own
 * list copies. *slot receives the buffer number. ZCG_EBUSY if the consumer has not
 * released that buffer since its last use (nothing is enqueued then).
 */
int zcg_pipeline_submit(zcg_pipeline* p, const int64_t* idx_host, int64_t n_idx, int* slot);
/*
 * Same, but a producer thread sleeps until the consumer thread releases the buffer:
 * timeout_ms < 0 waits without limit, otherwise ZCG_ETIMEDOUT after that long
 * (0 behaves like zcg_pipeline_submit). This is the back-pressure of the paper's
 * bounded queue between producer and consumer.
 */
int zcg_pipeline_submit_wait(zcg_pipeline* p, const int64_t* idx_host, int64_t n_idx,
                             int timeout_ms, int* slot);
/* Producer: no further minibatch will come; wakes a consumer blocked in next. */
int zcg_pipeline_finish(zcg_pipeline* p);
/*
 * Consumer: the next submitted minibatch, in submission order. Sleeps until one is
 * there (timeout_ms as above: ZCG_ETIMEDOUT); ZCG_ECLOSED once the producer has
 * finished and every minibatch has been handed out. Follow with acquire / release.
 */
int zcg_pipeline_next(zcg_pipeline* p, int timeout_ms, int* slot);
/* Consumer: make consumer_stream wait for that gather; yields the buffer and its row count.
 * ZCG_EINVAL for a slot that holds no submitted, unreleased minibatch. */
int zcg_pipeline_acquire(zcg_pipeline* p, int slot, void* consumer_stream, void** out_dev,
                         int64_t* n_rows);
/* Consumer: work enqueued so far on consumer_stream is the last that reads the buffer. */
int zcg_pipeline_release(zcg_pipeline* p, int slot, void* consumer_stream);
/* Waits for the gather stream, frees what the pipeline owns (never the output buffers).
 * No other thread may still be inside a call on p. */
int zcg_pipeline_destroy(zcg_pipeline* p);

/* Pinned host scratch for callers without another allocator (staging buffers). */
int zcg_pinned_alloc(int64_t bytes, void** host_ptr);
int zcg_pinned_free(void* host_ptr);

/* Library version, "major.minor". */
const char* zcg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ZCGATHER_H */
