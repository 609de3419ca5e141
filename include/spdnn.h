/* spdnn -- layer-by-layer sparse-DNN inference on one AMD MI355X (gfx950).
 *
 * The library evaluates, for l = 0 .. L-1,
 *
 *     Y_{l+1}[r][j] = min(max( sum_{k<32} Y_l[r][idx_l[j][k]] * val_l[j][k] + bias[j], 0), 32)
 *
 * (Section II-A-1, Eq. 1, with the clipped ReLU defined next to it; the steps
 * are those of Alg. 1, step 3), where Y_l is a dense batch x N feature map,
 * one feature row per input, and output neuron j of layer l has exactly 32
 * stored connections (input column idx_l[j][k], weight val_l[j][k]) -- or any
 * number of them for models built with spdnn_create_csr.  After
 * every layer the rows with no strictly positive output are dropped and the
 * list of surviving rows is compacted, as the host loop of Listing 1 does; a
 * dropped row is never evaluated again, which is exact because every bias is
 * required to be <= 0 (a zero row then stays zero).
 *
 * All entry points return 0 (SPDNN_OK) or a negative error code; none throws or
 * aborts.  spdnn_last_error() gives the message of the calling thread's last
 * failure.  Device memory is never allocated here: the caller passes arenas
 * (for example torch tensors) and keeps them alive while the handle uses them.
 * Everything runs on the HIP stream given to spdnn_create, on the device that
 * is current when the calls are made.
 */
#ifndef SPDNN_H
#define SPDNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spdnn_model* spdnn_t; /* opaque; owns small host metadata, two HIP events and a
                                        pinned host array of L+1 counters, nothing the caller allocated */

enum {
    SPDNN_OK = 0,
    SPDNN_EINVAL = -1, /* null pointer, N not a multiple of 4 in [32, 65536], L < 1, batch < 0,
                          misaligned buffer, column index outside [0, N) */
    SPDNN_EBIAS = -2,  /* some bias[j] > 0 or not finite: dropping all-zero rows would not be exact */
    SPDNN_EHIP = -3,   /* a HIP runtime call failed; message in spdnn_last_error() */
    SPDNN_ESIZE = -4   /* an arena is smaller than spdnn_weights_bytes / spdnn_work_bytes says */
};

enum { SPDNN_HOST = 0, SPDNN_DEVICE = 1 }; /* where the arrays given to spdnn_create live */

/* Bytes of device memory spdnn_create needs for a model of L layers of N neurons
 * (re-laid weights of all layers, bias, and staging for one raw layer), whatever the
 * sparsity patterns are.  The weights are held in the compact form whose footprint
 * Section III-B-2 discusses (16-bit column index + 32-bit value per connection, stored
 * lane-major as the transposed sliced-ELL of Section III-A-3) plus the tiling structures
 * of Section III-A-2.  Patterns whose 1024-neuron blocks each touch a narrow range of
 * input columns need less: see spdnn_weights_bytes_for_window. */
int spdnn_weights_bytes(int32_t N, int32_t L, size_t* bytes);

/* Same, for a model in which the input columns used by any block of 1024 consecutive
 * output neurons span at most widest_window columns (as spdnn_scan_windows reports).  The
 * tiling of Section III-A-2 stages a block's column range through LDS 4096 columns at a
 * time; ranges of 2 or more stages use a larger weight layout, which this accounts for.
 * spdnn_create accepts any arena of at least this size; with a smaller one than
 * spdnn_weights_bytes says it still works for every pattern, but layers with wider ranges
 * than the arena was sized for run a slower kernel. */
int spdnn_weights_bytes_for_window(int32_t N, int32_t L, int32_t widest_window, size_t* bytes);

/* The column footprint that the shared-memory tiling of Section III-A-2 stages per block of
 * output neurons, measured over the whole model: the
 * widest column range (in columns) of any 1024-neuron block of any layer -- when N is a
 * multiple of 2048, of any aligned pair of such blocks, which is what layers that run two
 * neurons per lane use.  idx as for spdnn_create.  scratch_dev: device memory, 256-byte aligned, at least N*32*4 + 2*N/128 +
 * 1024 bytes, contents scratch.  Blocks until done.  SPDNN_EINVAL on a column outside [0, N). */
int spdnn_scan_windows(int32_t N, int32_t L, const int32_t* const* idx, int32_t where, void* scratch_dev,
                       size_t scratch_bytes, void* hip_stream, int32_t* widest_window);

/* Bytes of device memory spdnn_infer needs for up to max_batch rows: two feature
 * maps of max_batch x N floats (the ping-pong pair of Listing 1; Section III-B's
 * footprint discussion counts the same two buffers) plus the row lists (`category`,
 * `globalcategories` of Listing 1) and the per-row activity flags (`active`). */
int spdnn_work_bytes(int32_t N, int32_t max_batch, size_t* bytes);

/* Build a model: once per network, outside inference time, like the tiling
 * structures of Section III-A-2, which are also built before inference and reused
 * by every call.
 *   idx, val : host arrays of L pointers.  idx[l][j*32+k] = input column of the k-th
 *              connection of output neuron j of layer l, in [0, N); val[l][j*32+k] its
 *              weight.  Duplicated columns within a neuron are allowed (they add up).
 *              The L pointers point to host memory if where == SPDNN_HOST, to device
 *              memory if where == SPDNN_DEVICE.  Read during the call only.
 *   bias     : N floats (host or device as `where` says), one per output neuron, the
 *              same for every layer (Listings 1 and 2 index it by output neuron);
 *              every entry must be <= 0.
 *   weights_arena : device memory, 256-byte aligned, >= spdnn_weights_bytes(N, L) or
 *              >= spdnn_weights_bytes_for_window(N, L, w) for the model's widest window w;
 *              owned by the caller, used by the handle until spdnn_destroy.
 *   hip_stream : a hipStream_t (NULL = default stream) on which create and infer enqueue.
 * On failure *out is NULL. */
int spdnn_create(spdnn_t* out, int32_t N, int32_t L, const int32_t* const* idx,
                 const float* const* val, const float* bias, int32_t where,
                 void* weights_arena, size_t weights_arena_bytes, void* hip_stream);

/* General sparse layers (Section II-A-1: W_l may be any sparse matrix; Listing 1 holds it in
 * CSR): output neuron j of layer l owns entries ptr[l][j] .. ptr[l][j+1]-1 of idx[l] / val[l],
 * any number of them, none included (its output is then the clipped bias, 0).  The library
 * evaluates
 *
 *     Y_{l+1}[r][j] = min(max( sum_k Y_l[r][idx_l[k]] * val_l[k] + bias[j], 0), 32)
 *
 * over the neuron's entries k.  A layer whose longest neuron has K <= 32 connections runs as
 * one launch of the fused kernel, shorter neurons padded with zero weights.  With K > 32 a
 * neuron is spread over one lane per 32 connections (K <= 8192); the lanes of a workgroup are
 * ordered by length, a wave runs only the steps its longest lane needs (the padding of Section
 * III-A-3, per wave), and the lanes' sums are added inside the workgroup before bias and ReLU.
 * Such a layer runs as up to P launches, P = ceil(K/32) rounded up to a power of two, each of
 * which computes the outputs of a share of the neurons and takes one layer's room in the
 * weights arena; P is what is called the layer's passes here.
 *
 * spdnn_csr_passes: passes[l] (host, may be NULL) = passes of layer l, *total = their sum,
 * which is the "L" to size the weights arena with (spdnn_weights_bytes(N, *total, ...)); if
 * widest_window is not NULL, also the widest column window of any 1024-neuron block (as
 * spdnn_scan_windows reports it) for spdnn_weights_bytes_for_window(N, *total, *widest_window).
 *   ptr        : host array of L pointers to device arrays of N+1 int32, ptr[l][0] >= 0,
 *                non-decreasing.
 *   idx        : as for spdnn_create_csr; may be NULL if widest_window is NULL.
 *   scratch_dev: device memory, 8-byte aligned, >= 8*L + 8*ceil(N/1024) bytes, contents scratch.
 * Blocks until done.  SPDNN_EINVAL if a ptr array decreases or is negative, or if a neuron has
 * more than 8192 connections. */
int spdnn_csr_passes(int32_t N, int32_t L, const int32_t* const* ptr, const int32_t* const* idx,
                     void* scratch_dev, size_t scratch_bytes, void* hip_stream, int32_t* passes,
                     int32_t* total, int32_t* widest_window);

/* Build a model of L general layers.  ptr, idx, val: host arrays of L pointers to DEVICE
 * arrays (ptr[l]: N+1 int32 as above; idx[l], val[l]: at least ptr[l][N] entries, columns in
 * [0, N), repeated columns add up); bias: N floats in DEVICE memory, all <= 0.  All read
 * during the call only.  weights_arena: device, 256-byte aligned, >= spdnn_weights_bytes(N,
 * total passes) (or the _for_window variant).  Everything else as spdnn_create; the handle is
 * used with the same spdnn_infer. */
int spdnn_create_csr(spdnn_t* out, int32_t N, int32_t L, const int32_t* const* ptr,
                     const int32_t* const* idx, const float* const* val, const float* bias,
                     void* weights_arena, size_t weights_arena_bytes, void* hip_stream);

/* Out-of-core weights (Section III-B-1): the re-laid weights of all layers live in host memory;
 * the device keeps the bias, two layer-sized buffers and the set-up staging area.  While layer l
 * runs from one buffer, a second HIP stream (made by the library, default priority) copies layer
 * l+1 into the other; a buffer is refilled as soon as the kernels that read it are done.
 *
 * spdnn_ooc_bytes: sizes of the two arenas for a model whose widest column window is
 * widest_window (as spdnn_scan_windows reports; N is always enough).
 * spdnn_create_ooc: as spdnn_create, with
 *   device_arena : device memory, 256-byte aligned, >= *device_bytes;
 *   host_arena   : host memory, 16-byte aligned, >= *host_bytes, written during the call and read
 *                  by every spdnn_infer; pinned memory (hipHostMalloc) lets the copies overlap the
 *                  kernels, pageable memory works but serialises them.
 * Both stay the caller's and must outlive the handle.  spdnn_infer is called as usual and gives
 * bit-identical results; it returns with the copy stream idle. */
int spdnn_ooc_bytes(int32_t N, int32_t L, int32_t widest_window, size_t* device_bytes,
                    size_t* host_bytes);
int spdnn_create_ooc(spdnn_t* out, int32_t N, int32_t L, const int32_t* const* idx,
                     const float* const* val, const float* bias, int32_t where,
                     void* device_arena, size_t device_arena_bytes, void* host_arena,
                     size_t host_arena_bytes, void* hip_stream);

/* Run all L layers on `batch` feature rows.
 *   Y0_dev : device, batch x N floats, row-major (row r = input r), 16-byte aligned, finite
 *            values; not modified.
 *   work_arena : device memory, 256-byte aligned, >= spdnn_work_bytes(N, batch); contents
 *            are scratch.
 *   n_active_host   : host int32, receives the number of rows of Y_L that have a strictly
 *            positive element (Alg. 1 step 4 works from these rows).
 *   active_rows_dev : device int32[batch]; first n_active entries = original row numbers of
 *            those rows, ascending.
 *   Y_final_dev : device float[batch*N] or NULL; row i of the first n_active rows is row
 *            active_rows[i] of Y_L.  NULL skips this output.
 * The call enqueues on the model's stream and returns after the stream has drained (it
 * must hand back n_active).  batch == 0 is valid and gives n_active = 0.  Calls on one
 * handle must not overlap. */
int spdnn_infer(spdnn_t h, const float* Y0_dev, int32_t batch, void* work_arena,
                size_t work_arena_bytes, int32_t* n_active_host, int32_t* active_rows_dev,
                float* Y_final_dev);

/* spdnn_infer for callers that cannot allocate device memory and have no work arena to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * results as spdnn_infer, but the work memory is a fixed array of SPDNN_STATIC_SCRATCH_BYTES bytes
 * that the library keeps in the memory of every GPU it runs on, from the time the library is loaded
 * until the process ends.  The call allocates nothing (no hipMalloc, no hipFree, no allocating
 * library routine) and fails with SPDNN_ESIZE, before any GPU work, when spdnn_work_bytes(N, batch)
 * exceeds the array (with N = 1024: up to about 8000 rows).  All handles and all calls on one GPU
 * share the array, and it keeps the last call's contents (every call re-initialises the lists, flags
 * and counters it reads): calls that overlap in time on one GPU race, on the same handle or on
 * different ones, also with different streams -- serialise them.  Inputs and outputs remain the
 * caller's. */
#define SPDNN_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int spdnn_infer_static(spdnn_t h, const float* Y0_dev, int32_t batch, int32_t* n_active_host,
                       int32_t* active_rows_dev, float* Y_final_dev);

/* Inputs that stay in host memory, handed to the GPU in serial batches (Section III-B-2: the
 * feature maps of all inputs need not fit the device; a batch is copied in while the one before
 * it is being inferred).  Y0_host: batch x N floats in host memory, row-major, read during the
 * call only; pinned memory (hipHostMalloc) lets the copies overlap the kernels, pageable memory
 * works but serialises them.  rows_per_batch >= 1 rows go through the layers at a time.
 *   work_arena : device memory, 256-byte aligned, >= spdnn_host_work_bytes(N, rows_per_batch):
 *            two input buffers of rows_per_batch x N floats plus what spdnn_infer needs for
 *            rows_per_batch rows; contents are scratch.
 *   n_active_host, active_rows_dev (capacity batch), Y_final_dev (capacity batch*N, or NULL): as
 *            for spdnn_infer, over the whole input -- rows are numbered as in Y0_host and come out
 *            ascending.
 * Results are those of one spdnn_infer over all rows (rows are independent, Eq. 1).  The copies
 * run on a second HIP stream that the handle makes on first use (default priority); the call
 * returns with both streams idle.  batch == 0 is valid. */
int spdnn_host_work_bytes(int32_t N, int32_t rows_per_batch, size_t* bytes);
int spdnn_infer_host(spdnn_t h, const float* Y0_host, int32_t batch, int32_t rows_per_batch,
                     void* work_arena, size_t work_arena_bytes, int32_t* n_active_host,
                     int32_t* active_rows_dev, float* Y_final_dev);

/* Release the handle (NULL is a no-op): the end of the life of the structures that
 * Section III-A-2 builds once per network.  The arenas stay the caller's. */
int spdnn_destroy(spdnn_t h);

/* Message of the last failure on the calling thread ("" if none).  Library plumbing; no
 * counterpart in the paper. */
const char* spdnn_last_error(void);

/* Measurement aid (not part of the paper's method): with profiling on, spdnn_infer brackets
 * every layer's fused launches (one, or one per pass of a general layer) with HIP events on the
 * model's stream. */
int spdnn_set_profiling(spdnn_t h, int32_t on);

/* After an spdnn_infer with profiling on: *layers_run = number of layers that were launched
 * (inference stops early once no row is active); for l < min(cap, *layers_run),
 * rows_in[l] = rows active on entry to layer l and fused_ms[l] = duration of that layer's
 * fused SpMM+bias+ReLU kernel (of all its passes, and of any wait for out-of-core weights) in
 * milliseconds.  Either array may be NULL. */
int spdnn_get_profile(spdnn_t h, int32_t cap, int32_t* layers_run, int32_t* rows_in,
                      float* fused_ms);

/* Measurement and test aid: which of the library's fused kernels layer l runs on, chosen at
 * spdnn_create from the layer's pattern (Section III-A-2's shared-memory stages) and weights:
 * SPDNN_KERNEL_SINGLE  every 1024-neuron block's column window fits one LDS stage;
 * SPDNN_KERNEL_STAGED  two stages (or a wider pattern that does not fit the wide format);
 * SPDNN_KERNEL_WIDE    three or more stages;
 * SPDNN_KERNEL_PAIR    one stage, every connection of the layer has the same weight and N is a
 *                      multiple of 2048: two output neurons per lane;
 * SPDNN_KERNEL_WIDE_PAIR  the same for five to eight stages;
 * SPDNN_KERNEL_WIDE_PAIR4 the same for two to four stages (the step lists of all stages stay in
 *                      registers).
 * SPDNN_KERNEL_ROW2    one weight, N a multiple of 4096, windows wider than one stage but every
 *                      4096-neuron unit within 16384 columns: four neurons per lane, tiles of two rows.
 * Returns SPDNN_EINVAL for a NULL handle or pointer or l outside [0, L). */
/* (A layer of several passes reports the kernel of its first pass.) */
#define SPDNN_KERNEL_SINGLE 0
#define SPDNN_KERNEL_STAGED 1
#define SPDNN_KERNEL_WIDE 2
#define SPDNN_KERNEL_PAIR 3
#define SPDNN_KERNEL_WIDE_PAIR 4
#define SPDNN_KERNEL_WIDE_PAIR4 5
#define SPDNN_KERNEL_ROW2 6
int spdnn_layer_kernel(spdnn_t h, int32_t l, int32_t* kind);

/* Whether spdnn_infer on `batch` rows runs all layers of the model in ONE launch (*yes = 1) or one launch
 * per layer (0).  One launch is taken for models of at most 1024 neurons per layer (one workgroup then
 * computes every neuron of its rows, so Listing 1's loop over the layers -- kernel, pruning, buffer swap
 * -- can run inside the workgroup) whose layers all fit one LDS stage, when a workgroup's share of the
 * rows is small (at most 128): the case in which the gaps between dependent kernels outweigh the
 * kernels.  With profiling on, such a launch's duration is shared out among the layers in proportion
 * to the rows they had (spdnn_get_profile). */
int spdnn_one_launch(spdnn_t h, int32_t batch, int32_t* yes);

/* Number of fused-kernel launches (passes) layer l takes: 1, or for a general layer whose
 * longest neuron has K > 32 connections ceil(K/32) rounded up to a power of two. */
int spdnn_layer_passes(spdnn_t h, int32_t l, int32_t* passes);

#ifdef __cplusplus
}
#endif
#endif /* SPDNN_H */
