/*
 * libbittrain -- the sparse bitmap activation codec of BitTrain on one MI355X.
 *
 * The format (Section 3.2, "Bitmap Format"): an activation tensor of n
 * elements, flattened in place, is stored as
 *   (i)  a bitmap with one bit per element, set where the element is non-zero;
 *   (ii) the non-zero elements, in ascending flattened index order.
 * Compression runs in the forward pass (Algorithm 1), restoration in the
 * backward pass (Algorithm 2).  The footprint is M_b = width * nnz + n / 8
 * bytes against M_d = width * n dense.
 *
 * Conventions fixed here where the paper is silent:
 *   - "zero" is the all-zero bit pattern of the element.  -0.0, NaNs, denormals
 *     and infinities are kept as values, so Algorithm 2 after Algorithm 1
 *     reproduces the tensor bit for bit.  fp16 and bf16 are the same codec.
 *   - element i owns bit (i mod 32), least significant first, of the uint32
 *     word (i div 32).  The bitmap has ceil(n/32) words; the unused high bits
 *     of the last word are written as 0, so popcount(bitmap) == nnz.
 *   - a cleared bit restores +0 (all-zero bits) of the element width.
 *   - tensors are flat, contiguous buffers; the shape stays with the caller.
 *
 * Every pointer named d_* is DEVICE memory owned by the caller.  The library
 * allocates nothing, frees nothing and never synchronises: each device call
 * enqueues its kernel(s) on `stream` and returns.  Argument errors are found on
 * the host before anything is launched; nothing is written in that case.
 * No exceptions, no errno, no logging: the return code is the only channel.
 */
#ifndef BITTRAIN_H
#define BITTRAIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BT_F32 = 0,  /* 4-byte elements */
    BT_F16 = 1,  /* 2-byte elements */
    BT_BF16 = 2, /* 2-byte elements; identical to BT_F16 at the byte level */
    BT_F64 = 3   /* 8-byte elements (the paper's formats are half, single and double precision) */
} bt_dtype;

typedef enum {
    BT_OK = 0,
    BT_ERR_NULL = 1,      /* a required pointer is NULL */
    BT_ERR_DTYPE = 2,     /* dtype is not one of bt_dtype */
    BT_ERR_ALIGN = 3,     /* a pointer is not aligned as documented */
    BT_ERR_WORKSPACE = 4, /* workspace smaller than bt_workspace_bytes(n, dtype) */
    BT_ERR_HIP = 5,       /* the HIP runtime refused the launch */
    BT_ERR_SIZE = 6,      /* n is beyond BT_MAX_ELEMENTS, or a size the call does not take */
    BT_ERR_UNSUPPORTED = 7 /* the call exists only in another build of the library */
} bt_status;

/* Largest number of tensors in one batched call. */
#define BT_MAX_BATCH 64

/* Largest n any call accepts (2^37 elements). */
#define BT_MAX_ELEMENTS ((uint64_t)1 << 37)

/* A hipStream_t, passed as an opaque pointer so that this header needs no HIP
 * header.  NULL is the default stream. */
typedef void *bt_stream;

/* ---- host-only, pure functions (no device is touched) -------------------- */

/* M_b of Section 3.2, generalised to the element width and to whole 32-bit
 * bitmap words: 4 * ceil(n/32) + nnz * sizeof(dtype).  Equals the paper's
 * 4 * nnz + n / 8 for fp32 whenever 32 divides n (every row of Table 1).
 * Returns 0 for an unknown dtype or nnz > n. */
size_t bt_compressed_size(uint64_t n, uint64_t nnz, bt_dtype dtype);

/* M_d of Section 3.2: n * sizeof(dtype), the dense footprint.  0 for an unknown dtype. */
size_t bt_dense_size(uint64_t n, bt_dtype dtype);

/* M_c of Section 3.2, the footprint of the coordinate-list (COO) format the paper
 * compares with: (sizeof(dtype) + index_bytes * ndim) * nnz, index_bytes being 4
 * (integer indices) or 8 (long indices).  0 for an unknown dtype, ndim == 0 or
 * another index size. */
size_t bt_coo_size(uint64_t nnz, uint32_t ndim, uint32_t index_bytes, bt_dtype dtype);

/* 4 * ceil(n/32): the bytes d_bitmap must hold. */
size_t bt_bitmap_bytes(uint64_t n);

/* Bytes of scratch that bt_compress / bt_decompress need for a tensor of n
 * elements: a 256-byte header plus 24 bytes per tile of the single-pass grid
 * scan (a tile is 32 KiB of dense data: 4096 eight-byte, 8192 four-byte or 16384
 * two-byte elements), in blocks of 256 tiles.  Monotone in n; 0 for an unknown dtype. */
size_t bt_workspace_bytes(uint64_t n, bt_dtype dtype);

/* Size in bytes of one element, 0 for an unknown dtype. */
size_t bt_dtype_size(bt_dtype dtype);

const char *bt_status_str(bt_status status);

/* ---- device calls -------------------------------------------------------- */

/* What a caller may look at, or set, in a workspace: 32-bit words at the start of it.
 *   BT_WS_ERROR_WORD        0 in normal operation.  The one wait inside the kernels that can
 *                           fail, the grid scan waiting for the counts of a call's tiles, is
 *                           bounded; a kernel whose wait ran out sets this word to 1 and
 *                           ends normally, staying inside all buffers (read it with
 *                           bt_workspace_status).  The outputs of that call are not valid (nnz
 *                           in particular is not written), and later calls on the workspace
 *                           write nothing at all, until bt_workspace_init has been run on it again.
 *   BT_WS_WAIT_LIMIT_WORD   passes of the grid scan after which it gives up; 0 (the initial
 *                           state) means the built-in limit of 2^20, far beyond what any
 *                           tensor needs.  Written by the caller only (a device-side store
 *                           or copy ordered before the call); meant for tests of the
 *                           failure path.
 *   BT_WS_PATIENCE_WORD     polls after which a tile's workgroup stops waiting for the grid
 *                           scan and counts what lies before its tile itself, from the
 *                           bitmap (restoration) or the input (compression): correct, only
 *                           slower; looked at every 256th poll; 0 means the built-in 4096.  Written by the caller only,
 *                           like the wait limit; meant for tests of that path.
 *   BT_WS_WIDE_WORD         non-zero: the grid scan of a call on one tensor writes every tile's
 *                           offset with 8-byte stores, which it otherwise does only once the
 *                           offsets reach 2^32 (below that it writes two neighbours' lower
 *                           halves in one store).  Same results; written by the caller only;
 *                           meant for tests of the wide path on tensors of ordinary size. */
#define BT_WS_ERROR_WORD 2
#define BT_WS_WAIT_LIMIT_WORD 3
#define BT_WS_PATIENCE_WORD 4
#define BT_WS_WIDE_WORD 5

/* Put a workspace into its initial state (all zero bytes) by enqueueing a fill
 * kernel on `stream`.  Required once after allocating a workspace, before its
 * first use, and again if a kernel using it was aborted.  After that the
 * kernels leave the workspace ready for the next call themselves, so
 * bt_compress and bt_decompress are one launch each.
 * d_workspace: 128-byte aligned.  Errors: BT_ERR_NULL, BT_ERR_ALIGN, BT_ERR_HIP. */
bt_status bt_workspace_init(void *d_workspace, size_t workspace_bytes, bt_stream stream);

/* Algorithm 1 (dense -> bitmap), as one fused pass over the input.
 *   d_in        n elements of `dtype`, 16-byte aligned, read once.
 *   d_bitmap    ceil(n/32) uint32 words, 4-byte aligned; every word is written.
 *   d_values    room for values_cap elements, element-aligned; on return
 *               elements [0, min(nnz, values_cap)) hold the non-zero elements in
 *               index order; the rest is untouched.
 *   values_cap  capacity of d_values in elements.  If nnz > values_cap nothing
 *               is written beyond the capacity, the bitmap and *d_nnz are still
 *               complete, and the caller sees the overflow as *d_nnz > values_cap.
 *               The worst case is n.
 *   d_nnz       one uint64, 8-byte aligned, written by the kernel: valid once
 *               `stream` has reached this call.
 *   d_workspace bt_workspace_bytes(n, dtype) bytes, 128-byte aligned, initialised
 *               once with bt_workspace_init.  A workspace must not be shared by
 *               two calls that can be in flight at the same time: calls that use
 *               one workspace must be ordered (same stream, or events).
 * Input and outputs must not overlap.  Algorithm 1's last step, giving up the
 * dense tensor, is the caller dropping d_in after this call is enqueued.  n == 0 only writes *d_nnz = 0.
 * Errors: BT_ERR_NULL, BT_ERR_DTYPE, BT_ERR_ALIGN, BT_ERR_SIZE, BT_ERR_WORKSPACE,
 * BT_ERR_HIP. */
bt_status bt_compress(const void *d_in, uint64_t n, bt_dtype dtype,
                      uint32_t *d_bitmap, void *d_values, uint64_t values_cap,
                      uint64_t *d_nnz,
                      void *d_workspace, size_t workspace_bytes, bt_stream stream);

/* bt_compress for callers that cannot allocate device memory and have no workspace to pass: code
 * whose stream is being recorded into a HIP graph, tight serving loops, harnesses that forbid
 * allocation.  Same arguments and results as bt_compress, without the workspace: the library
 * uses a workspace of its own, a device array of 256 + 6144 * BT_STATIC_MAX_TILES / 256 bytes
 * (393,472) that exists once on every GPU the library is loaded on until the process ends.  The
 * call allocates and frees nothing; it enqueues a fill kernel that clears that workspace and then
 * the compression kernel.
 *   n           at most BT_STATIC_MAX_TILES tiles (bt_tile_elems(dtype) elements each),
 *               else BT_ERR_SIZE.
 * All calls on one GPU share the one array: two of them that can be in flight at the same time
 * (different streams without an event between them) race, and so do the processes' threads that
 * issue them.  Errors: as bt_compress, without BT_ERR_WORKSPACE; BT_ERR_HIP also if the array's
 * address cannot be had. */
#define BT_STATIC_MAX_TILES 16384
bt_status bt_compress_static(const void *d_in, uint64_t n, bt_dtype dtype,
                             uint32_t *d_bitmap, void *d_values, uint64_t values_cap,
                             uint64_t *d_nnz, bt_stream stream);

/* Activation pruning (Section 4.3) fused into Algorithm 1: one pass that stores an
 * element only where its value exceeds `threshold` and treats it as zero elsewhere
 * (the paper's thresholds are 0, 0.01, 0.05 and 0.1).  The comparison is strict and exact:
 * an element is kept where its value, as a real number, is greater than `threshold`, as a
 * real number.  (BT_F64 elements are compared in double precision; narrower ones, widened
 * exactly, in single precision with the largest single at or below `threshold`, which
 * decides the same.)  A NaN element exceeds nothing and is dropped; a NaN threshold drops
 * everything.  The result is exactly bt_compress of the pruned tensor (so a +0.0
 * that survives a negative threshold is still not stored).  The bitmap marks the kept
 * elements, d_values holds their original
 * bit patterns in index order, *d_nnz their number.  With threshold 0 on a
 * pre-activation tensor x this is compress(ReLU(x)) without ever writing ReLU(x):
 * bt_decompress then yields ReLU(x) and bt_relu_backward_from_bitmap its backward.
 * All arguments, requirements and errors as for bt_compress. */
bt_status bt_compress_pruned(const void *d_in, uint64_t n, bt_dtype dtype, double threshold,
                             uint32_t *d_bitmap, void *d_values, uint64_t values_cap,
                             uint64_t *d_nnz,
                             void *d_workspace, size_t workspace_bytes, bt_stream stream);

/* The activation itself and its stash in one pass: as bt_compress_pruned, and in addition
 * the dense pruned tensor goes to d_dense_out (n elements, 16-byte aligned):
 *   d_dense_out[i] = x[i] where x[i] > threshold, +0 elsewhere,
 * i.e. y = ReLU(x) for threshold 0 -- what the next layer consumes -- while bitmap, values
 * and nnz are the compressed form of that same y, kept for the backward pass.  One read of
 * x serves both; run separately, ReLU and bt_compress read the activation three times and
 * write it once more.  d_dense_out may be d_in itself (in place) but must not partly
 * overlap it or any other argument.  Everything else as bt_compress_pruned. */
bt_status bt_activation_compress(const void *d_in, uint64_t n, bt_dtype dtype, double threshold,
                                 void *d_dense_out,
                                 uint32_t *d_bitmap, void *d_values, uint64_t values_cap,
                                 uint64_t *d_nnz,
                                 void *d_workspace, size_t workspace_bytes, bt_stream stream);

/* Algorithm 2 (bitmap -> dense).
 *   d_bitmap    ceil(n/32) words as written by bt_compress (bits at positions
 *               >= n are ignored).
 *   d_values    the non-zero elements in index order, popcount(bitmap) of them,
 *               element-aligned.  nnz is not an argument: it is implied by the
 *               bitmap, so no host synchronisation is needed between the two calls.
 *   d_out       n elements, 16-byte aligned; every element is written (values at
 *               set bits, +0 at cleared bits).
 *   d_workspace as for bt_compress.
 * Errors: as bt_compress. */
bt_status bt_decompress(const uint32_t *d_bitmap, const void *d_values, uint64_t n,
                        bt_dtype dtype, void *d_out,
                        void *d_workspace, size_t workspace_bytes, bt_stream stream);

/* ---- Algorithm 2 without the scan: the tile index ------------------------------
 *
 * Algorithm 2 carries one counter, j, the position in d_values of the next value.
 * bt_decompress has to find j for every tile of the tensor by a scan over the whole
 * bitmap before a tile can fetch its values.  bt_compress knows these numbers when it
 * writes the values: bt_compress_indexed also leaves them in d_index, entry t being j
 * at element t * bt_tile_elems(dtype) (the number of values stored before that
 * element), and bt_decompress_indexed starts every tile from its entry: no workspace,
 * no dependency between tiles.  The index is 8 bytes per 32 KiB of dense data, derived
 * from the bitmap alone; the compressed form proper (bitmap, values, nnz) is unchanged. */

/* Elements per tile: 32 KiB / sizeof(dtype).  0 for an unknown dtype. */
size_t bt_tile_elems(bt_dtype dtype);

/* Bytes d_index must hold: 8 * ceil(n / bt_tile_elems(dtype)). */
size_t bt_index_bytes(uint64_t n, bt_dtype dtype);

/* bt_compress, plus d_index (8-byte aligned, bt_index_bytes(n, dtype) bytes; every entry
 * is written).  Everything else as bt_compress. */
bt_status bt_compress_indexed(const void *d_in, uint64_t n, bt_dtype dtype,
                              uint32_t *d_bitmap, void *d_values, uint64_t values_cap,
                              uint64_t *d_nnz, uint64_t *d_index,
                              void *d_workspace, size_t workspace_bytes, bt_stream stream);

/* Algorithm 2 with j taken from the tile index.
 *   d_values, values_cap   the stored values and how many elements d_values holds (at
 *                          least the number of set bits, for a correct result); nothing at
 *                          or beyond values_cap is read, whatever d_index says.
 *   d_index                as written by bt_compress_indexed for this bitmap.  Entries that
 *                          do not belong to the bitmap give a wrong d_out, never an access
 *                          outside the buffers.
 * d_bitmap, d_out, alignment and errors as bt_decompress (no workspace errors). */
bt_status bt_decompress_indexed(const uint32_t *d_bitmap, const void *d_values, uint64_t values_cap,
                                const uint64_t *d_index, uint64_t n, bt_dtype dtype, void *d_out,
                                bt_stream stream);

/* Backward of y = ReLU(x) from the bitmap of y alone.  Algorithm 1 sets bit i
 * exactly where y[i] != 0, i.e. where x[i] > 0, which is the ReLU derivative, so
 * the values array is not needed:
 *   grad_in[i] = bit(i) ? grad_out[i] : +0      (a select, never a multiply).
 *   d_grad_out, d_grad_in   n elements each, 16-byte aligned; they may be the
 *                           same buffer (in place) but must not partly overlap.
 * Errors: BT_ERR_NULL, BT_ERR_DTYPE, BT_ERR_ALIGN, BT_ERR_SIZE, BT_ERR_HIP. */
bt_status bt_relu_backward_from_bitmap(const uint32_t *d_bitmap, const void *d_grad_out,
                                       uint64_t n, bt_dtype dtype, void *d_grad_in,
                                       bt_stream stream);

/* Double-mask batch normalisation (Section 3.1, "Exploiting Sparsity"): the sparsity
 * pattern of a normalisation layer's input is applied to its output, so that the
 * output compresses as well as the input did.  d_bitmap is the bitmap of that input
 * (as written by bt_compress), d_in the layer's output:
 *   out[i] = bit(i) ? in[i] : +0.
 * The same select as bt_relu_backward_from_bitmap, under the name of this use; all
 * requirements and errors as there (d_out may be d_in). */
bt_status bt_mask_apply(const uint32_t *d_bitmap, const void *d_in, uint64_t n, bt_dtype dtype,
                        void *d_out, bt_stream stream);

/* ---- many tensors in one launch ------------------------------------------------
 *
 * A training step stores every layer's activation (Section 3.2 applies the format
 * to all of them; Table 1 lists a network's layers).  Compressing them one call
 * each pays one launch and one pipeline fill-and-drain per tensor, which dominates
 * for the small layers; the batched calls run Algorithm 1 / Algorithm 2 on all the
 * tensors of a list in one launch per BT_MAX_BATCH tensors (restoration) or 52 tensors
 * (compression, whose items are larger).  The result for each
 * tensor is exactly what the single-tensor call gives.  The item arrays are HOST
 * memory and are read before the call returns; the pointers inside them are device
 * pointers with the meaning, alignment and overlap rules of the single-tensor calls.
 * All tensors of a call share one dtype. */

typedef struct {
    const void *d_in;    /* n elements, 16-byte aligned (may be NULL when n == 0) */
    uint64_t n;
    uint32_t *d_bitmap;  /* ceil(n/32) words */
    void *d_values;      /* room for values_cap elements */
    uint64_t values_cap;
    uint64_t *d_nnz;     /* one uint64 per tensor, 8-byte aligned, required also when n == 0 */
    uint64_t *d_index;   /* NULL, or bt_index_bytes(n, dtype) bytes, 8-byte aligned: the tensor's tile index,
                            as bt_compress_indexed writes it */
    void *d_dense_out;   /* bt_compress_batch_pruned only, else NULL: the dense pruned tensor, as
                            bt_activation_compress writes it (n elements, 16-byte aligned, may be d_in);
                            given for every tensor of the call that has elements, or for none */
} bt_compress_item;

typedef struct {
    const uint32_t *d_bitmap;
    const void *d_values;
    uint64_t n;
    void *d_out;         /* n elements, 16-byte aligned */
    uint64_t values_cap; /* bt_decompress_batch_indexed only: elements d_values holds, as for bt_decompress_indexed */
    const uint64_t *d_index; /* bt_decompress_batch_indexed only: the tensor's tile index */
} bt_decompress_item;

/* Workspace bytes a batched call on tensors of n[0..count) elements needs (host
 * function; n is a host array).  Never less than bt_workspace_bytes(0, dtype); 0 for
 * an unknown dtype or n == NULL with count != 0. */
size_t bt_batch_workspace_bytes(const uint64_t *n, size_t count, bt_dtype dtype);

/* Algorithm 1 on every tensor of items[0..count).  All items are checked before
 * anything is launched.  d_workspace: bt_batch_workspace_bytes(...) bytes, 128-byte
 * aligned, initialised once with bt_workspace_init; the same workspace may serve
 * single-tensor and batched calls alike, in stream order.  count == 0 does nothing.
 * d_index of an item, if
 * given, receives that tensor's tile index.  Errors: as bt_compress (the first offending item
 * decides); BT_ERR_NULL also if an item has d_dense_out. */
bt_status bt_compress_batch(const bt_compress_item *items, size_t count, bt_dtype dtype,
                            void *d_workspace, size_t workspace_bytes, bt_stream stream);

/* bt_compress_pruned on every tensor of items[0..count), one threshold for all; where the
 * items give d_dense_out, bt_activation_compress (the activations of a whole list of layers
 * pruned, handed on and stashed in one launch).  Otherwise as bt_compress_batch.
 * Errors: also BT_ERR_NULL if some tensors with elements have d_dense_out and others do not. */
bt_status bt_compress_batch_pruned(const bt_compress_item *items, size_t count, bt_dtype dtype,
                                   double threshold,
                                   void *d_workspace, size_t workspace_bytes, bt_stream stream);

/* Algorithm 2 on every tensor of items[0..count); otherwise as bt_compress_batch and
 * bt_decompress.  values_cap and d_index of the items are not looked at. */
bt_status bt_decompress_batch(const bt_decompress_item *items, size_t count, bt_dtype dtype,
                              void *d_workspace, size_t workspace_bytes, bt_stream stream);

/* bt_decompress_indexed on every tensor of items[0..count), each from the tile index that
 * bt_compress_indexed or a batched compression with d_index left for it: no scan, no
 * workspace, no dependency between tiles or tensors.  Errors: as bt_decompress_indexed. */
bt_status bt_decompress_batch_indexed(const bt_decompress_item *items, size_t count, bt_dtype dtype,
                                      bt_stream stream);

/* What became of the calls on a workspace, without knowing its layout: enqueues a kernel
 * that writes d_status[0] = 1 if a kernel gave up a wait on this workspace (the outputs of
 * that call and of every later one are not valid, and the workspace refuses work until
 * bt_workspace_init has been run on it again), else 0, and d_status[1] = the number of calls
 * completed on it since it was initialised.  d_status: two uint32 of device memory, valid
 * once `stream` has reached this call.  Errors: BT_ERR_NULL, BT_ERR_ALIGN, BT_ERR_HIP. */
bt_status bt_workspace_status(const void *d_workspace, uint32_t *d_status, bt_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* BITTRAIN_H */
