/*
 * pygraph_hip.h -- C ABI of libpygraph_hip: capture a chain of short GPU kernels once into a
 * hipGraph and replay it with fresh inputs, on one MI355X (gfx950).
 *
 * The problem (paper, Sec. 2.1-2.2): an iteration launches hundreds of short dependent kernels;
 * launching each from the CPU leaves the GPU idle, a graph replays them with one dispatch, but a
 * graph freezes kernel arguments at capture.  Three ways to give a replay its fresh inputs:
 *   - PG_GRAPH_COPY      copy every external input into a static placeholder the graph reads
 *                        (Sec. 2.2 "Cost-benefit analysis", Sec. 4 "Graph-Capture Layer");
 *   - PG_GRAPH_INDIRECT  Parameter Indirection (Sec. 3, Sec. 4 "Kernel generation"): kernels take
 *                        a pointer to a pointer, the replay rewrites 8 bytes per input;
 *   - selection          Selective graphs (Sec. 3, Sec. 4.3): per graph (here: per segment of the
 *                        chain) keep the fastest of {no graph, graph, graph + indirection}.
 *
 * Conventions
 *   - Every function returns a pg_status (0 = success), never aborts, never throws.  The text of
 *     the last error of the calling thread is pg_last_error(); the last HIP error code is
 *     pg_last_hip_error().
 *   - Pointers marked [dev] are device addresses, [host] host addresses.  The CALLER owns all
 *     device memory: external inputs, weights and one workspace blob.  The library borrows them,
 *     carves the workspace (placeholders, internal buffers, pointer table, copy job list; each
 *     sub-buffer 256-byte aligned), and allocates or frees no device memory itself.  It owns only
 *     host objects (descriptors, graphs, pinned staging).
 *   - Weights and the workspace must stay alive and unmoved until pg_chain_destroy.  External
 *     tensors must stay alive until the stream has finished the call that received them.  Freeing
 *     one earlier is the dangling-capture crash the paper describes (Sec. 1); it is not detected.
 *   - Calls that take a stream only enqueue work on it; the caller synchronises.  The stream
 *     must be a created (non-NULL) stream that is not capturing.  hip_stream is a hipStream_t.
 *   - External inputs are read-only to the chain; a kernel writes internal buffers only.
 *   - A chain object is not thread-safe; distinct chains may be used from distinct threads.
 */
#ifndef PYGRAPH_HIP_H
#define PYGRAPH_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PG_OK = 0,
    PG_EINVAL = 1,   /* bad argument or malformed descriptor */
    PG_ESTATE = 2,   /* call out of order (replay before capture, ...) */
    PG_EHIP = 3,     /* a HIP call failed; code in pg_last_hip_error() */
    PG_ENOMEM = 4,   /* workspace too small */
    PG_EUNAVAIL = 5  /* the mode does not exist for this segment */
} pg_status;

typedef enum { PG_F32 = 0, PG_BF16 = 1 } pg_dtype;

/* The chain's kernels.  fp32 arithmetic inside, one rounding to the storage dtype at the store. */
typedef enum {
    PG_ADD = 0,             /* o[i] = a[i] + b[i mod m]                                   */
    PG_MUL = 1,             /* o[i] = a[i] * b[i mod m]                                   */
    PG_GELU = 2,            /* o[i] = a[i] * Phi(a[i]), Phi the normal CDF (erf form)     */
    PG_RMSNORM = 3,         /* o[r,i] = x[r,i] * rsqrt(mean_i x[r,i]^2 + eps) * g[i]      */
    PG_GEMV = 4,            /* y[r,j] = sum_i W[j,i] * h[r,i]; W row-major [n, cols]      */
    PG_SCALE_BIAS_RELU = 5  /* o[b,c,p] = max(0, x[b,c,p]*s[c] + b[c]); x is [N,C,inner]  */
} pg_op;

/* Execution variants of a segment; the order is the tie-break order of pg_select. */
typedef enum { PG_EAGER = 0, PG_GRAPH_COPY = 1, PG_GRAPH_INDIRECT = 2 } pg_mode;

/* Where an operand lives (paper, Sec. 4 "Graph-Capture Layer": externally supplied parameters
 * need a refresh per replay, parameters produced inside the graph do not). */
typedef enum { PG_REF_NONE = 0, PG_REF_EXT = 1, PG_REF_INT = 2, PG_REF_WEIGHT = 3 } pg_ref_kind;

typedef struct { int32_t kind; int32_t index; } pg_ref;
typedef struct { int32_t dtype; int32_t reserved; int64_t numel; } pg_tensor_desc;

typedef struct {
    int32_t op;        /* pg_op */
    int32_t dtype;     /* pg_dtype of every operand and of the output */
    int32_t segment;   /* non-decreasing along the chain, starting at 0, no gaps */
    int32_t reserved;
    pg_ref out;        /* must be PG_REF_INT */
    pg_ref in[3];      /* ADD/MUL: a, b | GELU: a | RMSNORM: x, g | GEMV: W, h | SCALE_BIAS_RELU: x, s, b */
    int64_t n;         /* output elements (per row for RMSNORM and GEMV) */
    int64_t m;         /* ADD/MUL: period of b (0 means n); m <= numel(b) */
    int64_t rows;      /* RMSNORM/GEMV: batch rows */
    int64_t cols;      /* GEMV: input width; RMSNORM: hidden size (== n) */
    int64_t inner;     /* SCALE_BIAS_RELU: H*W; channels = numel(s) = numel(b); n % (channels*inner) == 0 */
    float eps;         /* RMSNORM */
    int32_t reserved2;
} pg_kernel_desc;

typedef struct pg_chain pg_chain;

typedef struct {
    int32_t n_kernels, n_segments, n_ext, n_ext_reading_kernels;
    int64_t copy_bytes_per_replay;   /* sum of external tensor bytes (payload of a copy refresh) */
    int64_t table_bytes_per_replay;  /* 8 * n_ext (payload of an indirect refresh)               */
    int64_t workspace_bytes;
    int32_t copy_chunks;             /* work items of the batched copy kernel                    */
    int32_t captured;                /* 1 after pg_capture                                       */
} pg_stats;

/* How pg_replay_indirect moves the pointers host -> device (paper, Sec. 4 "Graph-Capture
 * Layer": pointer copies are host-to-device transfers, unlike the device-to-device data copies). */
typedef enum {
    PG_TABLE_KERNARG = 0,      /* a one-wave kernel whose argument block carries the pointers          */
    PG_TABLE_MEMCPY = 1,       /* hipMemcpyAsync from a ring of pinned staging slots                   */
    PG_TABLE_GRAPH_MEMCPY = 2, /* the copy is the first node of the indirect graph itself: the host only
                                  fills pinned staging and launches the graph                         */
    PG_TABLE_HOST = 3          /* the table lives in pinned host memory: the host only writes it, the
                                  kernels' dereference crosses the host link                          */
} pg_table_refresh;
/* The last two read host memory when the graph runs, not when the call returns, so they alternate
 * between two instances (staging / table + graphs) and a call first waits, on the host, for the
 * replay that last used its instance; their graphs are built by the first indirect replay after
 * they are selected (which synchronises the stream and must not be captured). */

/* How a copy-mode replay moves the data of the external inputs into the placeholders (Sec. 2.2:
 * the deployed systems copy parameter by parameter; Sec. 5, table of bytes copied). */
typedef enum {
    PG_COPY_KERNEL = 0,    /* one batched copy kernel per <= 448 tensors (this library's design)  */
    PG_COPY_MEMCPY = 1     /* one device-to-device hipMemcpyAsync per tensor (the paper's baseline) */
} pg_copy_refresh;

/* Bytes of workspace [dev] a chain needs.  Host only.  The descriptor is validated as in
 * pg_chain_build as far as that is possible without the weight descriptors.  ext / ints: [host]
 * arrays of n_ext / n_int tensor descriptors. */
pg_status pg_chain_workspace_bytes(const pg_kernel_desc *kernels, int32_t n_kernels,
                                   const pg_tensor_desc *ext, int32_t n_ext,
                                   const pg_tensor_desc *ints, int32_t n_int, size_t *bytes_out);

/* Build a chain: validate the descriptor, lay out the workspace, resolve kernels and launch
 * shapes.  Host only: touches no device memory, makes no HIP call.
 *   kernels [host]         n_kernels descriptors, copied.
 *   weight_dev_ptrs [host] array of n_w device pointers [dev], each aligned to 16 bytes.
 *   workspace_dev [dev]    256-byte aligned, >= pg_chain_workspace_bytes; contents undefined.
 * Rules checked (PG_EINVAL otherwise): indices in range; sizes positive and consistent with the
 * tensor descriptors; every read of an internal buffer lies inside what an earlier kernel of the
 * chain wrote (so no state leaks from one replay into the next); out may alias in[0] exactly
 * (in-place) for ADD/MUL/GELU/SCALE_BIAS_RELU only and must not overlap any other operand. */
pg_status pg_chain_build(const pg_kernel_desc *kernels, int32_t n_kernels,
                         const pg_tensor_desc *ext, int32_t n_ext,
                         const pg_tensor_desc *ints, int32_t n_int,
                         const void *const *weight_dev_ptrs, const pg_tensor_desc *weights, int32_t n_w,
                         void *workspace_dev, size_t workspace_bytes, pg_chain **out);

/* Capture (paper, Sec. 2.2 stream capture; Sec. 4 "Graph-Capture Layer"): for every segment record
 * its kernels on `hip_stream` twice -- once reading the static placeholders, once reading the
 * pointer table -- instantiate and upload the graphs, and write the static part of the copy
 * kernel's job list into the workspace.  Synchronises the stream before returning.  Calling it
 * again re-captures: it first waits for everything queued on the device (a replay of the old graphs
 * may be running on any stream) and destroys the old graphs. */
pg_status pg_capture(pg_chain *chain, void *hip_stream);

/* One iteration, kernel by kernel from the host with the caller's pointers (the no-graph
 * baseline, Sec. 2.1).  ext_dev_ptrs [host]: n_ext device pointers [dev], each aligned to its
 * element size; 16-byte aligned pointers take the vector path. */
pg_status pg_eager(pg_chain *chain, const void *const *ext_dev_ptrs, void *hip_stream);

/* Kernels [k_begin, k_end) of the chain, launched eagerly as in pg_eager; internal buffers keep
 * whatever earlier calls left in them.  For stepping through a chain kernel by kernel (tests compare
 * each kernel's output with the CPU reference applied to that kernel's actual inputs). */
pg_status pg_eager_range(pg_chain *chain, const void *const *ext_dev_ptrs, int32_t k_begin, int32_t k_end,
                         void *hip_stream);

/* For callers that cannot allocate device memory or hand over a workspace: code that records the
 * chain into a HIP graph of its own, tight serving loops, harnesses that forbid hipMalloc.  One
 * eager pass of a chain (as pg_chain_build + pg_eager would run it) whose internal buffers live in a
 * static device array of PG_STATIC_SCRATCH_BYTES that the library's code object carries -- every GPU
 * the library runs on holds its own copy until the process ends.  The call allocates and frees no
 * device memory (no hipMalloc, hipFree, no allocating library routine); its host-side records are
 * kept from one call to the next and rebuilt only when the descriptor or the weight pointers change.
 *   kernels .. n_w        [host] the chain, as for pg_chain_build (same rules, same errors).  Only
 *                         the internal buffers are laid out: no placeholders, no pointer table.
 *   ext_dev_ptrs [host]   n_ext device pointers [dev], as for pg_eager.
 *   out_dev [dev]         receives the first out_bytes bytes of internal buffer out_int_index
 *                         (device-to-device, on the stream, after the last kernel); caller-owned.
 * Enqueues only; the caller synchronises.  The device the stream belongs to must be current.
 * Errors: PG_ENOMEM (nothing is launched) if the internal buffers, each aligned to 256 bytes, need
 * more than PG_STATIC_SCRATCH_BYTES; PG_EINVAL for a malformed descriptor, a bad output index, or
 * out_bytes beyond that buffer; PG_EHIP if the array's address cannot be resolved or a launch fails.
 * All calls on one GPU share that GPU's array, which keeps the last call's contents; nothing in it
 * has to start at zero (a pass overwrites every internal buffer before reading it).  Calls that
 * overlap in time on one GPU -- two streams, two threads -- race on it: serialise them. */
#define PG_STATIC_SCRATCH_BYTES (4u << 20)
pg_status pg_eager_static(const pg_kernel_desc *kernels, int32_t n_kernels,
                          const pg_tensor_desc *ext, int32_t n_ext,
                          const pg_tensor_desc *ints, int32_t n_int,
                          const void *const *weight_dev_ptrs, const pg_tensor_desc *weights, int32_t n_w,
                          const void *const *ext_dev_ptrs,
                          int32_t out_int_index, void *out_dev, size_t out_bytes, void *hip_stream);

/* One iteration: one launch of the batched copy kernel (external tensors -> placeholders, device
 * to device), then one graph launch per segment (Sec. 4 "Graph-Capture Layer", baseline). */
pg_status pg_replay_copy(pg_chain *chain, const void *const *ext_dev_ptrs, void *hip_stream);

/* One iteration: write the n_ext pointers into the device-resident table (8 bytes each), then one
 * graph launch per segment; kernels dereference their table slots first (Sec. 3, Sec. 4). */
pg_status pg_replay_indirect(pg_chain *chain, const void *const *ext_dev_ptrs, void *hip_stream);

/* One iteration with neither copies nor indirection: a third graph per segment, built from explicit
 * kernel nodes with direct pointers, whose external-reading nodes get their argument blocks
 * rewritten from the host before every launch (hipGraphExecKernelNodeSetParams).  This is the
 * alternative the graph API itself offers to what Sec. 3 "Parameter Indirection" does on the
 * device: one host call per external-reading kernel and replay, instead of 8 bytes per external.
 * The first call builds and instantiates the graphs (it synchronises the stream and must not be
 * captured).  Two executable instances alternate, and before an instance is rewritten the call
 * waits on the host for that instance's previous launch to finish, so a rewrite never touches
 * arguments a running launch may still read.  Results are identical to the other modes'. */
pg_status pg_replay_update(pg_chain *chain, const void *const *ext_dev_ptrs, void *hip_stream);

/* Selection rule (Sec. 4.3): mode_out[s] = the available variant of least cost, each segment on
 * its own.  cost_us [host] is [n_seg][3] in pg_mode order; a non-finite entry marks a variant that
 * does not exist; ties keep the earlier mode.  A negative cost or a segment with no variant is
 * PG_EINVAL.  Pure function: no chain, no device, deterministic. */
pg_status pg_select(const double *cost_us, int32_t n_seg, uint8_t *mode_out);

/* Slow-path profiler (Sec. 3 "Selective CUDA Graphs"): time every (segment, mode) on the given
 * inputs and fill cost_us_out [host] [n_seg][3] with the median microseconds over `iters`
 * samples (each sample: `inner` back-to-back runs then one stream synchronisation).  A segment
 * that reads no external operand reports PG_GRAPH_INDIRECT as NaN: it would be the same graph. */
pg_status pg_profile(pg_chain *chain, const void *const *ext_dev_ptrs, void *hip_stream,
                     int32_t iters, int32_t inner, double *cost_us_out);

/* The same slow-path measurement taken where the segment will run: between iterations of ANOTHER
 * chain (Sec. 4.3 measures each graph on its own; a server that alternates between the graphs of
 * several input shapes replays each one behind a different graph, with cold caches and a host that has
 * been busy with something else).  A sample is `inner` rounds of [one whole iteration of `background`
 * in background_mode (pg_mode), then the segment in the mode under test], one synchronisation at the
 * end, per round, minus the same for the background alone; cost_us_out [host] [n_seg][3] receives the
 * medians over `iters` samples (never below 0; NaN as in pg_profile).  Both chains must have been
 * captured (the background only if its mode is a graph mode) and are left with stale internal buffers. */
pg_status pg_profile_in_context(pg_chain *chain, const void *const *ext_dev_ptrs,
                                pg_chain *background, const void *const *background_ext_dev_ptrs, int32_t background_mode,
                                void *hip_stream, int32_t iters, int32_t inner, double *cost_us_out);

/* One iteration with a per-segment mode (mode [host], n_segments entries of pg_mode).  A copy-mode
 * segment refreshes the placeholders of the externals it reads; the pointer table is written once
 * per call if any segment is indirect.  PG_EUNAVAIL if a mode does not exist for its segment. */
pg_status pg_run_selected(pg_chain *chain, const uint8_t *mode, const void *const *ext_dev_ptrs,
                          void *hip_stream);

/* The two refresh steps on their own (what pg_replay_copy / pg_replay_indirect do before the
 * graph launches); for measuring the copy kernel and the table write in isolation. */
pg_status pg_refresh_copy(pg_chain *chain, const void *const *ext_dev_ptrs, void *hip_stream);
pg_status pg_refresh_indirect(pg_chain *chain, const void *const *ext_dev_ptrs, void *hip_stream);

/* Accessors.  Host only. */
pg_status pg_chain_int_buffer(const pg_chain *chain, int32_t int_index, void **dev_ptr_out, size_t *bytes_out);
/* The same under the name a caller looks for when it wants a result: a chain's outputs are the
 * internal buffers it designates. */
pg_status pg_chain_output(const pg_chain *chain, int32_t int_index, void **dev_ptr_out, size_t *bytes_out);
pg_status pg_chain_placeholder(const pg_chain *chain, int32_t ext_index, void **dev_ptr_out, size_t *bytes_out);
pg_status pg_chain_pointer_table(const pg_chain *chain, void **dev_ptr_out, size_t *bytes_out);
pg_status pg_chain_stats(const pg_chain *chain, pg_stats *out);
/* Launch shape of kernel `kernel` of the chain (workgroups, threads per workgroup): the same in every
 * replay mode, fixed by the kernel's shape alone at pg_chain_build.  Either output may be NULL. */
pg_status pg_chain_launch_shape(const pg_chain *chain, int32_t kernel, uint32_t *workgroups_out, uint32_t *threads_out);
pg_status pg_set_table_refresh(pg_chain *chain, int32_t how /* pg_table_refresh */);
pg_status pg_set_copy_refresh(pg_chain *chain, int32_t how /* pg_copy_refresh */);
/* Dispatch merging at capture (on by default).  A graph is "one dispatch, the GPU launches the rest"
 * (Sec. 2.2); on this machine every dependent kernel node still costs about 1.5 us of dispatch, so a
 * captured graph, which knows the whole chain, plays a run of up to 4 consecutive kernels with ONE
 * dispatch where it can: add / mul / GELU and RMSNorm over rows of 256 x 16 bytes, all element for
 * element over the same n elements (a whole number of 16-byte vectors; fp32 tensors of up to 16384
 * elements are worked one element per lane instead, with any n, and only there the fp32 GELU takes
 * part).  A lane runs the kernels in order on its elements with their stand-alone arithmetic and one
 * rounding each, stores every kernel's output that no later kernel of the run overwrites, and hands the stored
 * bits to the next kernel in registers, so
 * results stay bit-identical to eager launches.  A run ends where a kernel reads something an earlier
 * kernel of the run wrote in any other pattern than element for element.  Likewise up to 3 elementwise
 * kernels over the outputs of a bf16 GEMV over rows of 2048 columns (GELU of the result, the residual
 * add, an input add) ride in the GEMV's dispatch as an epilogue: each lane that holds a finished output
 * rounds it as the GEMV's store would and runs the following kernels on that element.  Up to 32 rows of
 * h the RMSNorm that produces the GEMV's input rides in front of it as a prologue (every workgroup
 * normalises the rows itself, one stores them); a run whose epilogue overwrites the buffer its prologue
 * reads writes a second copy of that buffer, which the workspace holds (pg_chain_workspace_bytes counts
 * it), and every segment ends with all internal buffers in their first copy, where pg_chain_int_buffer
 * and the other modes find them.  Outputs that a later kernel of the same run overwrites are not
 * stored (nothing could read them in between).  Eager launches are never merged.  `on` = 0 captures
 * one node per kernel.  Takes effect at the next pg_capture. */
pg_status pg_set_dispatch_merge(pg_chain *chain, int32_t on);
/* Kernel nodes that the graphs of one replay hold with merging on (*merged_out) and off
 * (*unmerged_out = the number of kernels).  Either output may be NULL.  Host only. */
pg_status pg_chain_graph_dispatches(const pg_chain *chain, int32_t *merged_out, int32_t *unmerged_out);
/* Destroys the graphs and host objects, after waiting for everything queued on the device the chain
 * was captured on (a graph still running, or a copy node still reading pinned staging, must not lose
 * them).  Device memory stays the caller's.  NULL is allowed. */
void pg_chain_destroy(pg_chain *chain);

const char *pg_last_error(void);
int pg_last_hip_error(void);
const char *pg_version(void);

#ifdef __cplusplus
}
#endif
#endif
