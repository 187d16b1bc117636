/*
 * compressed_layer.h - C ABI of the MI355X compressed-layer inference library.
 *
 * The library runs a fully-connected or convolutional layer directly from its
 * compressed form: pruned weights kept as relative-indexed entries per block,
 * value indices into a shared-weight codebook, and both entry arrays Huffman
 * coded (Sec. III-B and IV-A of "Efficient Inferencing of Compressed Deep Neural
 * Networks").  Decoding, codebook lookup and the sparse-weight x dense-activation
 * product all run in HIP kernels written for gfx950.
 *
 * Conventions
 *  - Plain C.  Every function returns an int32_t status: CL_OK (0) or a negative
 *    CL_E* code; cl_last_error() gives a thread-local message for the last
 *    failure on the calling thread.  Nothing aborts or throws across the ABI.
 *  - "host" pointers are ordinary CPU memory; "device" pointers (prefix d_) are
 *    GPU global memory of the current HIP device.  All tensors are owned by the
 *    caller; cl_layer handles are owned by the library and released with
 *    cl_layer_free().
 *  - Device entry points enqueue work on the given hipStream_t (passed as
 *    void*, NULL = the null stream) and return without synchronising.
 *  - Matrices are row-major.  W is M x K (outputs x inputs), activations are
 *    X[B][K] and Y[B][M] (one image per row).
 *  - Without a usable HIP device the device entry points fail with CL_EHIP; there
 *    is no CPU fallback.
 */
#ifndef COMPRESSED_LAYER_H
#define COMPRESSED_LAYER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CL_OK = 0,
    CL_EINVAL = -1,       /* bad argument (null pointer, size out of range, ...)   */
    CL_ENOMEM = -2,       /* host or device allocation failed                      */
    CL_ECORRUPT = -3,     /* a serialized layer failed validation                  */
    CL_EUNSUPPORTED = -4, /* valid request this build cannot serve                 */
    CL_EHIP = -5          /* a HIP runtime call failed / no device                 */
};

/* Bits per chunk of the compressed stream; the only value this build accepts. */
#define CL_CHUNK_BITS 4096
/* A chunk is up to 64 lane records of 64 bits, one per lane of a wavefront. */
#define CL_RECORD_BITS 64
#define CL_RECORDS_PER_CHUNK 64
/* A record holds at most this many entries (its count field has 4 bits). */
#define CL_MAX_RECORD_ENTRIES 15
/* Longest Huffman codeword the format allows. */
#define CL_MAX_CODE_LEN 12

/* Kernel selection for the forward entry points. */
enum {
    CL_PATH_AUTO = 0,     /* CL_PATH_SPARSE for up to 8 images and for blocks above      */
                          /*   128 x 128; else whichever of CL_PATH_MFMA_F32 and        */
                          /*   CL_PATH_SPARSE_WIDE the library's launch models price    */
                          /*   lower for this layer and batch (the dense tile multiplies */
                          /*   every zero of a block: at 9 % density the sparse product  */
                          /*   wins from about 100 images on, at 25 % it does not)       */
    CL_PATH_SPARSE = 1,   /* fused decode + sparse multiply on the vector ALUs      */
    CL_PATH_MFMA_F32 = 2, /* decode blocks to dense LDS tiles, fp32 MFMA; needs blocks */
                          /*   of at most 128 x 128, else CL_EUNSUPPORTED            */
    CL_PATH_MFMA_BF16 = 3,/* the same on the bf16 matrix cores: weights and activations */
                          /*   split into two bf16 terms each, three products per    */
                          /*   fp32 product, fp32 accumulation; error below 3 * 2^-16 */
                          /*   of sum |w x| per output; never picked by CL_PATH_AUTO  */
    CL_PATH_SPARSE_WIDE = 4 /* large batches on the vector ALUs: the sparse product of  */
                          /*   Algorithm 2 step 12 as written, one fp32 multiply-add   */
                          /*   per surviving weight and image, images across the lanes; */
                          /*   blocks of at most 128 x 128, else CL_EUNSUPPORTED.  One  */
                          /*   launch decodes the layer into a list of 4 bytes per      */
                          /*   surviving weight in the workspace, one multiplies it for */
                          /*   every tile of 64, 128 or 256 images (by batch).          */
                          /*   Run-to-run identical                                     */
};

/* How a weight matrix is compressed.
 *  M, K          W is M x K; the layer computes b = W a + v (Eq. 1-2).
 *  weight_bits   r: a value index has r bits, i.e. at most 2^r - 1 shared non-zero
 *                values plus the reserved index 0 (Sec. III-B; 5 for FC, 8 for
 *                CONV layers in Sec. V-A).  1..8.
 *  index_bits    k: a relative index has k bits; a run of more than 2^k - 1 zeros
 *                is broken by padding entries (Sec. III-B; 4 AlexNet, 5 VGG-16).
 *                1..8.
 *  block_h/w     bh x bw blocks, stored contiguously block after block in the
 *                order Algorithm 2 visits them (Sec. IV-A).  Inside a block the
 *                positions run along a row first (the 4 x 16 re-layout of the
 *                paper's 8 x 8 example), so the relative index is a column gap
 *                that carries over from one row of the block to the next; a block
 *                of one column, (M, 1), is a plain CSC column with a relative row
 *                index.  Edge blocks keep their true, smaller shape.
 *  chunk_bits    must be CL_CHUNK_BITS (0 is taken as that).
 *  max_code_len  limit on Huffman codeword length, 0 = CL_MAX_CODE_LEN; must be
 *                >= max(weight_bits, index_bits) and <= CL_MAX_CODE_LEN. */
typedef struct {
    int32_t M, K;
    int32_t weight_bits;
    int32_t index_bits;
    int32_t block_h, block_w;
    int32_t chunk_bits;
    int32_t max_code_len;
} cl_layer_desc;

typedef struct cl_layer cl_layer;

/* Size and content figures of a compressed layer. */
typedef struct {
    int64_t nnz;            /* surviving weights                                     */
    int64_t padding;        /* padding entries (value index 0)                       */
    int64_t entries;        /* nnz + padding                                         */
    int64_t n_blocks;
    int64_t n_chunks;
    int64_t val_bits;       /* Huffman-coded bits of the value-index array           */
    int64_t idx_bits;       /* Huffman-coded bits of the relative-index array        */
    int64_t val_bits_unlimited; /* same arrays under unrestricted Huffman codes:     */
    int64_t idx_bits_unlimited; /*   what the length limit costs                     */
    int64_t n_records;
    int64_t payload_bytes;  /* lane records (8 B each): counts, codewords, padding   */
    int64_t table_bytes;    /* chunk table + block_ptr + panel table                 */
    int64_t model_bytes;    /* payload + tables + codebook + code lengths: the bytes */
                            /*   a forward pass has to fetch                         */
    int64_t lut_bytes;      /* decode tables derived at load time (not stored)       */
    int32_t val_max_len, idx_max_len;
} cl_stats;

/* Layout of the compressed streams.
 *
 * The entries of a block are cut into lane records of 64 bits.  Bit b of a record
 * is bit b of its little-endian 64-bit word.
 *   bits [0, 4)   n, the number of entries in the record (1..15)
 *   from bit 4 upwards: the value-index codewords of those n entries, in entry
 *                 order, each codeword's bits in the order the code tree is walked
 *   from bit 63 downwards: the relative-index codewords of the same n entries
 *                 (the first bit of the first codeword is bit 63, the next bit 62, ...)
 *   the bits in between are zero.
 * So a record carries a span of the value-index stream and the matching span of
 * the relative-index stream, with both start addresses fixed by the layout - the
 * per-record form of the row_ptr 2-tuple of Sec. III-B.  A record never crosses a
 * block.
 *
 * A chunk is up to 64 consecutive records of one block (4096 bits when full): what
 * one wavefront decodes.  One table entry per chunk, plus a sentinel entry at index
 * n_chunks holding the totals:
 *   sym_off   index of the chunk's first entry ("symbol offset")
 *   rec_off   index of its first record (start address of the chunk in the stream)
 *   blk       the block all its entries belong to
 *   pos0      sum of (z + 1) over the entries of that block that precede the chunk,
 *             i.e. the carry of the position prefix sum (Algorithm 1 step 7)       */
typedef struct {
    uint32_t sym_off;
    uint32_t rec_off;
    uint32_t blk;
    uint32_t pos0;
} cl_chunk_meta;

/* Read-only view of the host copy of a layer, for inspection and tests.  The
 * pointers stay valid until cl_layer_free().
 *  val_code / idx_code   codeword of each symbol with bit j = the j-th bit of the
 *                        codeword in tree-walk order.                              */
typedef struct {
    cl_layer_desc desc;
    const float *codebook;         /* 2^r                                            */
    const uint8_t *val_len;        /* 2^r                                            */
    const uint32_t *val_code;      /* 2^r                                            */
    const uint8_t *idx_len;        /* 2^k                                            */
    const uint32_t *idx_code;      /* 2^k                                            */
    const uint32_t *block_ptr;     /* n_blocks + 1, entry offsets                    */
    const uint32_t *panel_chunk;   /* n_panels + 1, first chunk of each block row    */
    const cl_chunk_meta *chunk_meta; /* n_chunks + 1                                 */
    const uint64_t *records;       /* n_records                                      */
    int64_t n_blocks, n_chunks, n_records, n_entries;
    int32_t n_panels;
    const uint32_t *chunk_nz;      /* n_chunks + 1: entries that are not padding in all */
                                   /*   chunks before this one (derived at load time)  */
    int64_t max_block_nnz;         /* most surviving weights in one block              */
    int32_t max_group_blocks;      /* most blocks touched by the chunks c0 + 8 g ..    */
                                   /*   c0 + 8 g + 7 of a block row whose first chunk  */
                                   /*   is c0 (derived at load time)                   */
    /* Layers with blocks of at most 128 x 128 (else both null): the order in which the   */
    /* large-batch sparse path lists a block's surviving weights - those in the block's    */
    /* columns 0-63 first, then those in columns 64-127, each half row by row (derived at  */
    /* load time).                                                                         */
    const uint32_t *chunk_half;    /* 2 n_chunks: list position of the first surviving  */
                                   /*   weight of chunk c in half 0 (2c) and 1 (2c + 1) */
    const uint32_t *group_ptr;     /* n_blocks x 2 x 17: list position where rows 8q .. */
                                   /*   of half h of block b start ([b][h][q]); [16]:   */
                                   /*   where the half ends                             */
} cl_host_view;

const char *cl_last_error(void);

/* Sec. III-B pipeline on the host: quantise the surviving weights of W to the
 * codebook, build the relative-indexed entries block by block, Huffman-code both
 * arrays (length-limited, canonical) and lay the codewords out in lane records and
 * 4096-bit chunks with their chunk table.
 *  W_host      M*K fp32, already pruned: a pruned weight is exactly 0.  Non-finite
 *              values are rejected.
 *  codebook    2^r fp32 with codebook[0] == 0, or NULL for a linear codebook:
 *              2^r - 1 centres equally spaced between the smallest and largest
 *              surviving weight.  Each surviving weight takes the nearest centre
 *              (fp64 distance, ties to the lower index) among indices 1..2^r - 1.
 *  out         receives a new handle (host copy only; see cl_layer_upload).
 * Errors: CL_EINVAL for bad descriptors (including M*K or the entry count
 * exceeding 2^31 - 1), null pointers, non-finite weights, codebook[0] != 0. */
int32_t cl_compress_layer(const cl_layer_desc *desc, const float *W_host,
                          const float *codebook_or_null, cl_layer **out);

/* Copy the layer (payload, tables, codebook, decode tables) to the current HIP
 * device.  Synchronous.  Must precede any device entry point.  Idempotent. */
int32_t cl_layer_upload(cl_layer *layer);

int32_t cl_layer_free(cl_layer *layer);
int32_t cl_layer_stats(const cl_layer *layer, cl_stats *out);
int32_t cl_layer_host_view(const cl_layer *layer, cl_host_view *out);

/* Relocatable byte image of a layer (the paper's use case keeps many compressed
 * models resident, Sec. II).  Call with buf == NULL to get the size in *bytes;
 * then with a buffer of at least that size.  cl_layer_deserialize validates the
 * image completely (every chunk is decoded on the host) and returns CL_ECORRUPT
 * for anything inconsistent. */
int32_t cl_layer_serialize(const cl_layer *layer, void *buf, size_t *bytes);
int32_t cl_layer_deserialize(const void *buf, size_t bytes, cl_layer **out);

/* Algorithm 1 steps 5-8 / Algorithm 2 steps 5-9 on the GPU, for the whole layer:
 * Huffman-decode both arrays, prefix-sum the relative indices, look the values up
 * and arrange them.  Any output pointer may be NULL.
 *  d_val_sym, d_idx_sym   entries bytes each: the decoded value indices and
 *                         relative indices in entry order
 *  d_block_ptr            n_blocks + 1 uint32 entry offsets
 *  d_dense                M*K fp32, the matrix the layer multiplies by           */
int32_t cl_decode_layer(const cl_layer *layer, uint8_t *d_val_sym, uint8_t *d_idx_sym,
                        uint32_t *d_block_ptr, float *d_dense, void *stream);

/* Device scratch a forward call needs for (batch, path): the partial output tiles
 * of the workgroups of each block row and, on the MFMA paths, the activations in
 * the layout the kernel reads (transposed, K laid out block by block; two bf16
 * planes for CL_PATH_MFMA_BF16).  Needs a HIP device (CL_EHIP otherwise). */
int32_t cl_fc_workspace_bytes(const cl_layer *layer, int32_t batch, int32_t path, size_t *out);

/* The path a forward call with these arguments runs on: `path` itself unless it is
 * CL_PATH_AUTO, else the library's choice for this layer and batch on the current
 * device (see CL_PATH_AUTO).  Needs a HIP device (CL_EHIP otherwise). */
int32_t cl_fc_resolved_path(const cl_layer *layer, int32_t batch, int32_t path, int32_t *out);

/* Y = act(X W^T + v) straight from the compressed layer (Eq. 1-2 with the
 * decoding steps of Algorithm 2 fused in).
 *  d_X     batch x K fp32        d_bias  M fp32 or NULL
 *  d_Y     batch x M fp32, overwritten
 *  relu    non-zero applies max(0, .)
 *  path    CL_PATH_*.  CL_PATH_SPARSE takes up to 8 images per launch in a fixed
 *          summation order when block_h <= 256 (run-to-run identical); a launch for
 *          9-16 images at once, or a layer with taller blocks, adds lane sums into
 *          a shared LDS tile with floating-point atomics, so the last bits of Y can
 *          differ between runs.  The tiles of a block row are added up in a fixed
 *          order either way.  The other paths are run-to-run identical.
 *  d_workspace / workspace_bytes   at least cl_fc_workspace_bytes(); may be NULL
 *          when that is 0
 * Errors: CL_EINVAL (null pointers, batch < 1, workspace too small, layer not
 * uploaded), CL_EUNSUPPORTED (a dense-tile path with more than 2^21 images in one
 * call, or a launch of more than 2^31 - 1 workgroups) - nothing is launched then. */
int32_t cl_compressed_fc_forward(const cl_layer *layer, const float *d_X, const float *d_bias_or_null,
                                 float *d_Y, int32_t batch, int32_t relu, int32_t path,
                                 void *d_workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory or pass a workspace - code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc: the same call as
 * cl_compressed_fc_forward (same arguments, kernels, paths and results) with the scratch
 * in an array that is part of the library's device image, CL_STATIC_SCRATCH_BYTES per
 * GPU, held by every GPU the library runs on until the process ends.  The call allocates
 * and frees nothing; the array's address on a device is looked up once, when the first
 * layer is uploaded to that device.  A (layer, batch, path) whose
 * cl_fc_workspace_bytes() exceeds CL_STATIC_SCRATCH_BYTES is refused with
 * CL_EUNSUPPORTED and nothing is launched.  No kernel reads the scratch before writing
 * it, so nothing has to be cleared between calls; but every call on a GPU uses that
 * GPU's one array: calls that may overlap on one GPU (different streams, or host
 * threads) race and must be serialised by the caller. */
#define CL_STATIC_SCRATCH_BYTES (16u << 20)
int32_t cl_compressed_fc_forward_static(const cl_layer *layer, const float *d_X, const float *d_bias_or_null,
                                        float *d_Y, int32_t batch, int32_t relu, int32_t path, void *stream);

/* A stack of fully connected layers, layer i + 1 reading what layer i writes
 * (Eq. 1 applied layer after layer; the FC6-8 stack of Table IV): the same kernels
 * as cl_compressed_fc_forward, layer by layer on the given stream, with the
 * intermediate activations kept in the workspace.  Between two layers on the
 * dense-tile paths the finishing kernel writes the next layer's activations in the
 * layout its multiply kernel reads (when that layer has 128-column blocks and K a
 * multiple of 128), which saves the separate transposition; on the run-to-run
 * identical paths the results are the same bit for bit as those of per-layer calls,
 * and where a layer runs on CL_PATH_SPARSE they are, like that path's own results
 * from one call to the next, the same within the rounding of a different order of
 * additions (see cl_compressed_fc_forward), not bit for bit.  The workspace holds up to four
 * copies of each scratch buffer, used in rotation (a kernel that writes where
 * another has just read runs slower on this chip).
 *  layers          n_layers uploaded layers, layers[i]->K == layers[i-1]->M
 *  d_X             batch x layers[0]->K fp32
 *  d_bias_or_null  NULL, or n_layers device pointers (each M_i fp32 or NULL)
 *  d_Y             batch x layers[n_layers-1]->M fp32, overwritten
 *  relu_hidden     non-zero applies max(0, .) after every layer but the last
 *  relu_last       the same for the last layer
 *  path            CL_PATH_*, resolved per layer as in cl_compressed_fc_forward
 *  d_workspace     at least cl_fc_stack_workspace_bytes(), 256-byte aligned
 * Errors: CL_EINVAL (null pointers, n_layers < 1, layer sizes that do not chain,
 * workspace too small, a layer not uploaded) - nothing is launched then. */
int32_t cl_fc_stack_workspace_bytes(const cl_layer *const *layers, int32_t n_layers, int32_t batch, int32_t path,
                                    size_t *out);
int32_t cl_compressed_fc_stack_forward(const cl_layer *const *layers, int32_t n_layers, const float *d_X,
                                       const float *const *d_bias_or_null, float *d_Y, int32_t batch,
                                       int32_t relu_hidden, int32_t relu_last, int32_t path, void *d_workspace,
                                       size_t workspace_bytes, void *stream);

/* Several layers of one shape in one grid (Sec. V: requests for different models, or layers
 * whose inputs do not depend on each other, served together; Algorithm 2 per layer on the
 * small-batch kernel).  One launch does the decode-and-multiply of all n layers, one the
 * finishing - where n calls of cl_compressed_fc_forward pay 2 n launches and n times the
 * fixed part of a launch.
 * cl_layer_group_create: layers must be uploaded to the current device and agree in M, K,
 * block_h and block_w (CL_EINVAL otherwise); the group keeps the pointers, not the layers:
 * they must outlive it.  The group owns a small device table; free it with
 * cl_layer_group_free (NULL is allowed).
 * cl_compressed_fc_group_forward:
 *  batch           1 .. 16 images per layer (one batch tile of the small-batch kernel; more
 *                  is CL_EUNSUPPORTED)
 *  d_X             layer i's input, batch x K fp32, at d_X + i * x_stride (x_stride in
 *                  floats; 0: every layer reads the same input)
 *  d_bias_or_null  NULL, or layer i's M fp32 at d_bias + i * bias_stride (0: shared)
 *  d_Y             layer i's output, batch x M fp32, at d_Y + i * batch * M; overwritten
 *  d_workspace     at least cl_fc_group_workspace_bytes(), 256-byte aligned
 * Results as CL_PATH_SPARSE gives them (tolerance-identical from call to call).
 * Errors: CL_EINVAL, CL_EUNSUPPORTED, CL_EHIP - nothing is launched on the first two. */
typedef struct cl_layer_group cl_layer_group;
int32_t cl_layer_group_create(const cl_layer *const *layers, int32_t n_layers, cl_layer_group **out);
void cl_layer_group_free(cl_layer_group *group);
int32_t cl_fc_group_workspace_bytes(const cl_layer_group *group, int32_t batch, size_t *out);
int32_t cl_compressed_fc_group_forward(const cl_layer_group *group, const float *d_X, size_t x_stride,
                                       const float *d_bias_or_null, size_t bias_stride, float *d_Y, int32_t batch,
                                       int32_t relu, void *d_workspace, size_t workspace_bytes, void *stream);

/* Convolution geometry.  The layer's matrix has M = out_channels rows and
 * K = (C / groups) * R * S columns, row oc being filter oc flattened as
 * ((c * R + r) * S + s) (Sec. III-A: filters become rows, receptive fields
 * columns).  Output channel oc of group oc / (out_channels / groups) sees only
 * that group's input channels.  Zero padding. */
typedef struct {
    int32_t C, H, W;
    int32_t R, S;
    int32_t stride, pad, groups;
    int32_t out_channels;
} cl_conv_desc;

int32_t cl_conv_workspace_bytes(const cl_layer *layer, const cl_conv_desc *conv, int32_t batch,
                                int32_t path, size_t *out);
/* The least scratch cl_compressed_conv_forward works with.  Where the call would
 * keep the column matrices of all filter groups in the workspace (see below), it can,
 * given less than cl_conv_workspace_bytes() but at least this, take the filter groups
 * one after the other through the same buffers and decode the blocks inside the
 * multiply kernel - about half the memory for a layer with two filter groups, the same
 * results, more time (AlexNet conv2 at batch 1: 45 instead of 32 us).  Where the
 * call gathers the columns itself, nothing needs less and the two sizes are equal. */
int32_t cl_conv_workspace_bytes_min(const cl_layer *layer, const cl_conv_desc *conv, int32_t batch,
                                    int32_t path, size_t *out);

/* d_X: batch x C x H x W fp32 (NCHW); d_Y: batch x out_channels x P x Q fp32 with
 * P = (H + 2 pad - R) / stride + 1, Q likewise.  The convolution is the product of the
 * layer's matrix with the matrix whose columns are the receptive fields (Sec. III-A),
 * computed on an MFMA path, all filter groups in one launch, in one of two forms:
 *  - CL_PATH_MFMA_F32 from 512 columns (images x output pixels) on, when 128-column
 *    tiles give the chip enough to do (work items for a sixteenth of the compute units,
 *    block products for half): every block of the layer is decoded once per call into a
 *    dense 128 x 128 tile in the workspace (64 KiB per block), and the multiply kernel
 *    gathers each 128 x 128 piece of the column matrix from d_X into LDS itself - the
 *    column matrix is never written to memory.  Workspace: the decoded blocks, a row
 *    table (8 bytes per row of the layout), partial tiles when block rows are split.
 *    Needs R, S <= 32 and 129 images of input under 2^29 elements, else the other form.
 *  - otherwise the receptive fields are written out as columns in the workspace, one
 *    matrix per filter group and at most 1 GiB of them at a time (the batch is cut
 *    into image groups accordingly), and multiplied by the kernels of the FC paths,
 *    which decode the blocks for every tile of columns.  This is the form that
 *    cl_conv_workspace_bytes() sizes the workspace for in that case; with a workspace
 *    between cl_conv_workspace_bytes_min() and that, the compact form described there
 *    runs instead.
 * Below cl_conv_workspace_bytes_min() the call fails with CL_EINVAL.
 * path is CL_PATH_AUTO (= CL_PATH_MFMA_F32), CL_PATH_MFMA_F32 or
 * CL_PATH_MFMA_BF16, anything else is CL_EUNSUPPORTED, as are blocks above
 * 128 x 128, with groups > 1 a block_h that does not divide
 * out_channels / groups, more than 2^21 output pixels per image and image planes
 * of more than 2^30 pixels. */
int32_t cl_compressed_conv_forward(const cl_layer *layer, const cl_conv_desc *conv, const float *d_X,
                                   const float *d_bias_or_null, float *d_Y, int32_t batch, int32_t relu,
                                   int32_t path, void *d_workspace, size_t workspace_bytes, void *stream);

/* Variable batch sizes per layer (Sec. V-C): the dynamic program over
 * <layer, batch, reserved memory> that minimises time per image subject to
 * A + IN(i,B) + WS(i) + OUT(i,B) <= TOT and, optionally, a latency threshold.
 *  time_ms            n_layers x n_batches, Time(i, batch_set[j]), row-major
 *  batch_set          n_batches candidate batch sizes, ascending
 *  in/out_bytes_per_image  n_layers each (IN and OUT are linear in the batch)
 *  ws_bytes           n_layers
 *  mem_step_bytes     granularity of the reserved-memory axis; reservations round up
 *  latency_cap_ms     <= 0 means none
 *  out_batch_per_layer  n_layers; out_ms_per_image  the optimum, +inf (and
 *                     CL_EUNSUPPORTED) when no plan is feasible
 * Host only. */
int32_t cl_plan_batches(int32_t n_layers, const int32_t *batch_set, int32_t n_batches,
                        const double *time_ms, const int64_t *in_bytes_per_image,
                        const int64_t *out_bytes_per_image, const int64_t *ws_bytes,
                        int64_t tot_bytes, int64_t mem_step_bytes, double latency_cap_ms,
                        int32_t *out_batch_per_layer, double *out_ms_per_image);

/* The fixed-function layers between the convolutions of a whole network (the norm
 * and pool rows of Table IV; Sec. II: pooling layers "implement fixed functions"),
 * so that a network can run end to end on the device with per-layer batch sizes.
 * d_X: batch x C x H x W fp32 (NCHW), device.  Asynchronous on `stream`.  Neither call
 * works in place: d_Y must not overlap d_X (an output's inputs are read by other
 * workgroups than the one that writes it).
 *
 * cl_maxpool_forward: maximum over size x size windows at the given stride, no
 *   padding, windows fully inside the image; d_Y: batch x C x P x Q with
 *   P = (H - size) / stride + 1, Q likewise.
 * cl_lrn_forward: local response normalisation across channels,
 *   y[c] = x[c] / (k + alpha / n * sum of x[c']^2 over the n channels centred on c,
 *   clipped to [0, C))^beta; n odd; d_Y has the shape of d_X.  The sum and the power
 *   are taken in fp32; for a positive, normal, finite base the power is
 *   exp2(-beta * log2(base)), relative error near 1e-7 * (1 + |beta * log2(base)|).
 * Errors: CL_EINVAL (null pointers, non-positive sizes, window larger than the
 * image, even n), CL_EUNSUPPORTED (pooling with more than 2^30 outputs per plane,
 * normalisation with batch x ceil(C / 8) above 2^31 - 1) - nothing is launched then; CL_EHIP. */
int32_t cl_maxpool_forward(const float *d_X, float *d_Y, int32_t batch, int32_t C, int32_t H, int32_t W,
                           int32_t size, int32_t stride, void *stream);
int32_t cl_lrn_forward(const float *d_X, float *d_Y, int32_t batch, int32_t C, int32_t H, int32_t W,
                       int32_t n, float alpha, float beta, float k, void *stream);

/* Measurement hook for benchmarks (not part of the paper's method).  While
 * enabled, every forward call brackets the first launch of its main kernel (the
 * first batch tile; not the small reduction kernel) with a pair of HIP events on
 * the call's stream.  cl_last_kernel_ms() waits for the most recent bracket and
 * returns its duration in milliseconds and the number of launches it covered (1).
 * Process-wide state, not thread safe; leave it off in production. */
int32_t cl_set_kernel_timing(int32_t enable);
int32_t cl_last_kernel_ms(float *ms, int32_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* COMPRESSED_LAYER_H */
