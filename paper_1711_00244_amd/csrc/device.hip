// gfx950 kernels and their launchers: record-parallel Huffman decode, position
// prefix sums, codebook lookup, and the fused sparse-weight x dense-activation
// product (Algorithm 2 of the paper, re-cast for 64-lane wavefronts).
//
// One wavefront owns one chunk: up to 64 lane records of 64 bits, all of one block.
// Lane l reads record l with one 64-bit load (a full 512-byte burst per wavefront).
// A record holds n entries: their value-index codewords run up from bit 4, their
// relative-index codewords run down from bit 63, so a lane decodes both spans side
// by side from two shift registers with two decode tables held in LDS.
//   decode  both spans, entry by entry, symbols kept in registers, z + 1 summed per lane
//   scan    one wavefront prefix sum turns lane sums into each lane's starting
//           position (Algorithm 1 step 7) and lane counts into output slots
//   use     the entries in order, each with its position: store it (decode_layer),
//           multiply-accumulate it (sparse forward) or place it in a dense tile (MFMA forward)
//
// One translation unit: this file holds the host side (device image of a layer, launch
// shapes, the entry points) and includes the kernels - decode.hpp (wavefront primitives,
// decoding and placement passes), sparse_kernels.hpp, mfma_kernels.hpp, wide_kernels.hpp, bf16_kernels.hpp,
// conv_kernels.hpp, finish_kernels.hpp, layer_kernels.hpp.
#include <hip/hip_runtime.h>
#include <type_traits>

#include <algorithm>
#include <atomic>
#include <climits>
#include <cstdio>
#include <cstring>
#include <memory>
#include <vector>

#include "layer.hpp"

namespace cl {

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(CL_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// A launch of n workgroups along x; more than a grid holds is refused, not wrapped.
#define GRID_TRY(g, n)                                                                        \
    do {                                                                                      \
        const int64_t n_ = (n);                                                               \
        if (n_ < 1 || n_ > INT32_MAX) return fail(CL_EUNSUPPORTED, "a launch of %lld workgroups does not fit a grid", (long long)n_); \
        (g) = dim3((unsigned)n_);                                                             \
    } while (0)

constexpr int kWaves = 8;                 // wavefronts per workgroup
constexpr int kSparseChunksPerWave = 1;   // chunks a wavefront of the sparse kernel decodes, one after the other
                                          // (2 amortises the table copy but measured 18 % slower at batch 1)
constexpr int kThreads = kWaves * 64;

// Everything a kernel needs to read a layer, passed by value.
struct LayerDev {
    const uint64_t *records;
    const cl_chunk_meta *meta;
    const uint32_t *panel_chunk;
    const uint32_t *block_chunk;
    const uint32_t *chunk_nz;
    const uint32_t *chunk_half;          // null unless the blocks are at most 128 x 128 (with group_ptr)
    const uint32_t *group_ptr;
    const float *codebook;
    const lut_t *val_lut;
    const lut_t *idx_lut;
    int M, K, bh, bw, nbw;
    int val_bits, idx_bits, ncode;       // index widths of the decode tables, codebook entries
    int table_rows;                      // 16-byte rows of the table image (tables + codebook)
    uint32_t n_chunks;
    int panel0;                          // first block row of a launch that covers only some (a filter group); else 0
};

// Bytes of the table image: both decode tables, then the codebook, each padded to 16 bytes.
static size_t table_image_bytes(int vbits, int ibits, int ncode)
{
    const size_t tb = (((size_t)1 << vbits) + ((size_t)1 << ibits)) * sizeof(lut_t);
    return ((tb + 15) & ~(size_t)15) + (((size_t)ncode * 4 + 15) & ~(size_t)15);
}

static LayerDev make_dev(const cl_layer *L)
{
    LayerDev d;
    d.records = L->dev.records;
    d.meta = L->dev.meta;
    d.panel_chunk = L->dev.panel_chunk;
    d.block_chunk = L->dev.block_chunk;
    d.chunk_nz = L->dev.chunk_nz;
    d.chunk_half = L->dev.chunk_half;
    d.group_ptr = L->dev.group_ptr;
    d.codebook = L->dev.codebook;
    d.val_lut = L->dev.val_lut;
    d.idx_lut = L->dev.idx_lut;
    d.M = L->desc.M;
    d.K = L->desc.K;
    d.bh = L->desc.block_h;
    d.bw = L->desc.block_w;
    d.nbw = L->nbw;
    d.val_bits = L->val_lut_bits;
    d.idx_bits = L->idx_lut_bits;
    d.ncode = 1 << L->desc.weight_bits;
    d.table_rows = (int)(table_image_bytes(L->val_lut_bits, L->idx_lut_bits, d.ncode) / 16);
    d.n_chunks = (uint32_t)L->n_chunks;
    d.panel0 = 0;
    return d;
}

#include "decode.hpp"
#include "sparse_kernels.hpp"
#include "mfma_kernels.hpp"
#include "wide_kernels.hpp"
#include "bf16_kernels.hpp"
#include "conv_kernels.hpp"
#include "finish_kernels.hpp"
#include "layer_kernels.hpp"

// ------------------------------------------------------------------------- //
// host side
// ------------------------------------------------------------------------- //
struct DeviceLimits {
    int device = -1;
    int cus = 0;
    size_t max_lds = 0;
};

static int32_t device_limits(DeviceLimits &dl)
{
    static thread_local DeviceLimits cache;
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (cache.device != dev) {
        int cus = 0, lds = 0;
        HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        HIP_TRY(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
        cache.device = dev;
        cache.cus = cus;
        cache.max_lds = (size_t)lds;
    }
    dl = cache;
    return CL_OK;
}

// Event bracket around the main kernel of the last forward call (benchmarks only).
struct KernelTiming {
    bool on = false, valid = false;
    hipEvent_t a = nullptr, b = nullptr;
    int launches = 0;
};
static KernelTiming g_timing;

static void timing_begin(hipStream_t st)
{
    if (!g_timing.on) return;
    g_timing.launches = 0;
    g_timing.valid = hipEventRecord(g_timing.a, st) == hipSuccess;
}

static void timing_end(hipStream_t st, int launches)
{
    if (!g_timing.on || !g_timing.valid) return;
    g_timing.launches = launches;
    g_timing.valid = hipEventRecord(g_timing.b, st) == hipSuccess;
}

// Scratch for the entry point that may not allocate: one array per GPU, placed by the
// loader, held until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress; kernels get the address that call returns for the current
// device.
static __device__ __align__(256) unsigned char g_static_scratch[CL_STATIC_SCRATCH_BYTES];

constexpr int kMaxScratchDevices = 64;
static std::atomic<void *> g_static_scratch_ptr[kMaxScratchDevices];

// Address of the current device's copy of the scratch array (looked up once per device).
static int32_t static_scratch(void **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxScratchDevices) return fail(CL_EUNSUPPORTED, "device %d: static scratch is tracked for devices 0..%d", dev, kMaxScratchDevices - 1);
    void *p = g_static_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)));
        if (!p) return fail(CL_EHIP, "hipGetSymbolAddress gave a null address");
        g_static_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return CL_OK;
}

void release_device(cl_layer *L)
{
    if (L->dev.blob) {
        (void)hipFree(L->dev.blob);
        L->dev = DeviceImage{};
    }
}

static int32_t require_device(const cl_layer *L)
{
    if (!L) return fail(CL_EINVAL, "null layer");
    if (!L->dev.blob) return fail(CL_EINVAL, "layer is not on the device: call cl_layer_upload first");
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != L->dev.device) return fail(CL_EINVAL, "layer was uploaded to device %d, current device is %d", L->dev.device, dev);
    return CL_OK;
}

}  // namespace cl

using namespace cl;

extern "C" int32_t cl_layer_upload(cl_layer *L)
{
    if (!L) return fail(CL_EINVAL, "null layer");
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(CL_EHIP, "no HIP device");
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (L->dev.blob && L->dev.device == dev) return CL_OK;
    {
        // set-up time: find this device's copy of the static scratch array now, so that the
        // non-allocating entry point has nothing left to look up (a device beyond the
        // tracked range is refused there, not here)
        void *scratch = nullptr;
        if (dev >= 0 && dev < kMaxScratchDevices)
            if (int32_t rc = static_scratch(&scratch)) return rc;
    }
    release_device(L);
    struct Sec { const void *src; size_t bytes; size_t off; };
    // decode tables + codebook, laid out as in LDS
    const int ncode = 1 << L->desc.weight_bits;
    std::vector<char> image(table_image_bytes(L->val_lut_bits, L->idx_lut_bits, ncode), 0);
    {
        const size_t vb = L->val_lut.size() * sizeof(lut_t), ib = L->idx_lut.size() * sizeof(lut_t);
        std::memcpy(image.data(), L->val_lut.data(), vb);
        std::memcpy(image.data() + vb, L->idx_lut.data(), ib);
        std::memcpy(image.data() + ((vb + ib + 15) & ~(size_t)15), L->codebook.data(), L->codebook.size() * 4);
    }
    Sec secs[9] = {
        {L->records.data(), L->records.size() * 8, 0},
        {L->meta.data(), L->meta.size() * sizeof(cl_chunk_meta), 0},
        {L->block_ptr.data(), L->block_ptr.size() * 4, 0},
        {L->panel_chunk.data(), L->panel_chunk.size() * 4, 0},
        {image.data(), image.size(), 0},
        {L->block_chunk.data(), L->block_chunk.size() * 4, 0},
        {L->chunk_nz.data(), L->chunk_nz.size() * 4, 0},
        {L->chunk_half.data(), L->chunk_half.size() * 4, 0},
        {L->group_ptr.data(), L->group_ptr.size() * 4, 0},
    };
    size_t total = 0;
    for (auto &s : secs) { s.off = total; total += (s.bytes + 255) / 256 * 256; }
    total += 256;
    std::vector<char> host(total, 0);
    for (auto &s : secs)
        if (s.bytes) std::memcpy(host.data() + s.off, s.src, s.bytes);
    char *blob = nullptr;
    if (hipMalloc((void **)&blob, total) != hipSuccess) return fail(CL_ENOMEM, "hipMalloc of %zu bytes failed", total);
    if (hipMemcpy(blob, host.data(), total, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(blob);
        return fail(CL_EHIP, "hipMemcpy to device failed");
    }
    L->dev.device = dev;
    L->dev.blob = blob;
    L->dev.blob_bytes = total;
    L->dev.records = (const uint64_t *)(blob + secs[0].off);
    L->dev.meta = (const cl_chunk_meta *)(blob + secs[1].off);
    L->dev.block_ptr = (const uint32_t *)(blob + secs[2].off);
    L->dev.panel_chunk = (const uint32_t *)(blob + secs[3].off);
    L->dev.block_chunk = (const uint32_t *)(blob + secs[5].off);
    L->dev.chunk_nz = (const uint32_t *)(blob + secs[6].off);
    L->dev.chunk_half = L->group_ptr.empty() ? nullptr : (const uint32_t *)(blob + secs[7].off);
    L->dev.group_ptr = L->group_ptr.empty() ? nullptr : (const uint32_t *)(blob + secs[8].off);
    L->dev.val_lut = (const lut_t *)(blob + secs[4].off);
    L->dev.idx_lut = L->dev.val_lut + L->val_lut.size();
    L->dev.codebook = (const float *)(blob + secs[4].off + ((L->val_lut.size() + L->idx_lut.size()) * sizeof(lut_t) + 15) / 16 * 16);
    clear_error();
    return CL_OK;
}

extern "C" int32_t cl_decode_layer(const cl_layer *L, uint8_t *d_val_sym, uint8_t *d_idx_sym,
                                   uint32_t *d_block_ptr, float *d_dense, void *stream)
{
    if (int32_t rc = require_device(L)) return rc;
    hipStream_t st = (hipStream_t)stream;
    const LayerDev D = make_dev(L);
    if (d_block_ptr)
        HIP_TRY(hipMemcpyAsync(d_block_ptr, L->dev.block_ptr, (size_t)(L->n_blocks + 1) * 4, hipMemcpyDeviceToDevice, st));
    if (d_dense) {
        const size_t n = (size_t)L->desc.M * L->desc.K;
        hipLaunchKernelGGL(fill_kernel, dim3((unsigned)std::min<size_t>((n + 255) / 256, 4096)), dim3(256), 0, st, d_dense, n, 0.0f);
        HIP_TRY(hipGetLastError());
    }
    if (L->n_chunks > 0 && (d_val_sym || d_idx_sym || d_dense)) {
        const size_t lds = smem_fixed_bytes(D.val_bits, D.idx_bits, D.ncode);
        const dim3 grid((unsigned)((L->n_chunks + kWaves - 1) / kWaves));
        hipLaunchKernelGGL(decode_kernel, grid, dim3(kThreads), lds, st, D, d_val_sym, d_idx_sym, d_dense);
        HIP_TRY(hipGetLastError());
    }
    clear_error();
    return CL_OK;
}

namespace {

// Launch shape of the sparse forward path for one layer and batch.
struct SparsePlan {
    int bt_max = 1;          // batch tile of the main kernel (power of two, <= 16)
    int wg_per_panel = 0;    // workgroups per block row (8 wavefronts of kSparseChunksPerWave chunks each)
    int xwant = 0;           // activation columns to stage in LDS per image (3 blocks wide)
    size_t fixed = 0;        // LDS bytes of tables + codebook
    size_t part_bytes = 0;   // partial-tile buffer in the workspace
    int xcap_for(int bt) const { return (size_t)xwant * 4 * bt <= 32 * 1024 ? xwant : 0; }
    size_t lds_for(const cl_layer *L, int bt) const
    {
        const size_t tiles = private_tiles(L->desc.block_h, bt) ? kWaves : 1;
        return fixed + (tiles * L->desc.block_h + xcap_for(bt)) * 4 * bt;
    }
};

// (one_tile: the caller wants the whole batch, up to 16 images, in one batch tile)
int32_t plan_sparse(const cl_layer *L, int batch, size_t max_lds, SparsePlan &P, bool one_tile = false)
{
    P.fixed = table_image_bytes(L->val_lut_bits, L->idx_lut_bits, 1 << L->desc.weight_bits);
    P.xwant = (int)std::min<int64_t>(L->desc.K, (1 + 2 * kSparseChunksPerWave) * (int64_t)L->desc.block_w);
    // largest power-of-two batch tile (<= 16) that fits; prefer to stay under 64 KiB
    size_t budget = std::min<size_t>(max_lds, 64 * 1024);
    if (P.lds_for(L, 1) > budget) budget = max_lds;
    if (P.lds_for(L, 1) > budget) return fail(CL_EUNSUPPORTED, "block_h %d needs more LDS than a workgroup has", L->desc.block_h);
    // two launches with a tile per wavefront are faster than one of 16 images through atomics
    P.bt_max = !one_tile && private_tiles(L->desc.block_h, kPrivateTileBT) ? kPrivateTileBT : 16;
    while (P.bt_max > 1 && (P.lds_for(L, P.bt_max) > budget || P.bt_max / 2 >= batch)) P.bt_max >>= 1;
    P.wg_per_panel = (int)((L->max_panel_chunks + kWaves * kSparseChunksPerWave - 1) / (kWaves * kSparseChunksPerWave));
    P.part_bytes = (size_t)L->n_panels * P.wg_per_panel * L->desc.block_h * P.bt_max * sizeof(float);
    return CL_OK;
}

// Whether a stack could leave out the finishing kernel between two layers on this path,
// as far as this layer goes (as producer or consumer): the batch is a single batch tile,
// so that there is one set of partial tiles, and - for the consumer - every workgroup
// stages its activation columns in LDS, where the sum of the tiles is formed.
bool sparse_can_fold(const cl_layer *L, const SparsePlan &P, int batch)
{
    if (batch > P.bt_max || (batch & (batch - 1))) return false;
    const int64_t widest = std::min<int64_t>(L->desc.K, (int64_t)L->max_group_blocks * L->desc.block_w);
    return widest <= P.xcap_for(batch);
}

// Launch shape of the MFMA path.
struct MfmaPlan {
    int nq = 4;              // 32-image groups per workgroup tile
    bool bf16 = false;       // three bf16 products instead of one fp32 product
    int Bp = 0;              // batch rounded up to whole image tiles
    int splits = 1;          // workgroups sharing the blocks of one block row
    size_t lds = 0;
    size_t xt_bytes = 0, part_bytes = 0;
};

// columns per workgroup of the finishing kernel: as many as leave 1024 workgroups
int reduce_col_tile(int panels, int ncols)
{
    int ct = kColTile;
    while (ct > 1 && (int64_t)panels * ((ncols + ct - 1) / ct) < 1024) ct >>= 1;
    return ct;
}

// rows of the block-by-block activation layout, tail included
size_t xt_rows(const cl_layer *L) { return (size_t)L->nbw * kTile + kXtTailRows; }

// Most columns (images, or images x output pixels) of one dense-tile launch: keeps the
// kernels' 32-bit column arithmetic and the y extent of the layout kernels' grids in range.
constexpr int kMaxTileColumns = 1 << 21;

bool mfma_capable(const cl_layer *L) { return L->desc.block_h <= kTile && L->desc.block_w <= kTile; }

// Image tile, padded column count and split of the block rows for `ncols` columns and
// `panels` block rows, from a small model of a layer's launches with measured constants
// (cycles per workgroup: 12 k to start; per block 5 k of decoding and bookkeeping plus
// 4.1 k of multiplies per 32 columns of the tile - 1.5 k on the bf16 matrix cores;
// workgroups run in rounds of one per CU; and 3 cycles per 4 KB of partial tiles, which
// are written, flushed at the kernel's end and read again by the finishing kernel -
// 2 per 5 KB next to the gathered convolution's kernel, nothing where one workgroup per
// block row writes the output itself, `direct`).  Fitted
// to sweeps over every tile width and split of the AlexNet and VGG-16 FC layers at 8 to
// 1024 images: the choice is the fastest measured shape for the large layers and
// within 3 % of it on average for a 1000-row layer, where the partial tiles decide; for
// the gathered convolution, to sweeps over the splits of the AlexNet and VGG-16 layers
// at 2 to 128 images (0.2 % from the fastest on average, 5 % at worst).
void mfma_shape(const cl_layer *L, int panels, int ncols, int cus, bool bf16, int &nq, int &np, int &splits, bool gathered = false,
                bool direct = false, int64_t *cost = nullptr)
{
    cus = std::max(1, cus);
    nq = 0;
    int64_t best = -1;
    for (int q : {1, 2, 4, 8}) {
        if (gathered && 32 * q != kConvColumns) continue;      // conv_mfma_kernel has one tile width
        const int w = 32 * q;
        const int cols = (ncols + w - 1) / w * w;
        const int64_t tiles = (int64_t)panels * (cols / w);
        // any split up to three rounds of workgroups (eight for the gathered convolution,
        // whose long block rows gain from them): more, shorter workgroups can beat one
        // round that leaves CUs idle
        const int64_t max_rounds = gathered ? 8 : 3;
        const int sp_max = (int)std::max<int64_t>(1, std::min<int64_t>(L->nbw, (max_rounds * cus + tiles - 1) / tiles));
        for (int sp = 1; sp <= sp_max; ++sp) {
            const int64_t rounds = (tiles * sp + cus - 1) / cus;
            const int64_t blocks = (L->nbw + sp - 1) / sp;
            // blocks decoded beforehand: the gathering costs less than a decode
            int64_t t = gathered ? rounds * (8000 + blocks * (1500 + 4100 * q))
                              : rounds * (12000 + blocks * (5000 + (bf16 ? 1500 : 4100) * q));
            if (!(direct && sp == 1)) t += (int64_t)panels * sp * cols * L->desc.block_h * (int64_t)sizeof(float) * (gathered ? 2 : 3) / (gathered ? 5000 : 4000);
            if (best < 0 || t < best) {
                best = t;
                nq = q;
                np = cols;
                splits = sp;
            }
        }
    }
    if (cost) *cost = best;
}

size_t mfma_lds_bytes(const cl_layer *L, bool bf16)
{
    const size_t tables = table_image_bytes(L->val_lut_bits, L->idx_lut_bits, 1 << L->desc.weight_bits);
    return bf16 ? tables + 2 * (size_t)kBf16BufFloats * 4 + ((size_t)4 << L->desc.weight_bits) : tables + 2 * (size_t)kWTileBytes;
}

// bf16 elements of one plane of the split activations, read-ahead tail included
size_t xb_plane_elems(const cl_layer *L, int np) { return ((size_t)L->nbw * 8 + kXbTailGroups) * np * 16; }

// bytes of the activations as the dense-tile kernel of the given precision reads them
size_t xt_bytes_for(const cl_layer *L, int np, bool bf16)
{
    const size_t raw = bf16 ? 2 * xb_plane_elems(L, np) * sizeof(uint16_t) : xt_rows(L) * np * sizeof(float);
    return (raw + 255) / 256 * 256;
}

int32_t plan_mfma(const cl_layer *L, int batch, bool bf16, const DeviceLimits &dl, MfmaPlan &P)
{
    if (!mfma_capable(L)) return fail(CL_EUNSUPPORTED, "the MFMA path needs blocks of at most %d x %d", kTile, kTile);
    if (batch > kMaxTileColumns) return fail(CL_EUNSUPPORTED, "the dense-tile paths take at most %d images per call", kMaxTileColumns);
    P.bf16 = bf16;
    mfma_shape(L, L->n_panels, batch, dl.cus, bf16, P.nq, P.Bp, P.splits);
    P.lds = mfma_lds_bytes(L, bf16);
    if (P.lds > dl.max_lds) return fail(CL_EUNSUPPORTED, "the MFMA path needs %zu bytes of LDS", P.lds);
    P.xt_bytes = xt_bytes_for(L, P.Bp, bf16);
    P.part_bytes = (size_t)L->n_panels * P.splits * P.Bp * L->desc.block_h * sizeof(float);
    return CL_OK;
}

// Raises a kernel's dynamic LDS limit when a launch needs more than any before it on
// this device (the attribute sticks; asking again for every launch costs a runtime
// call each time).  `seen` belongs to one kernel instantiation.
constexpr int kMaxDevices = 64;
struct LdsLimit { std::atomic<size_t> bytes[kMaxDevices]; };

static int32_t ensure_lds(const void *kernel, size_t lds, LdsLimit &seen)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    const bool tracked = dev >= 0 && dev < kMaxDevices;
    if (tracked && seen.bytes[dev].load(std::memory_order_relaxed) >= lds) return CL_OK;
    HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    if (tracked) seen.bytes[dev].store(lds, std::memory_order_relaxed);
    return CL_OK;
}

template <int NQ>
int32_t launch_mfma_as(const LayerDev &D, int panels, int splits, int np, int panels_per_x, size_t x_stride, size_t lds,
                       const float *xt, float *part, const DirectOut &out, hipStream_t st)
{
    static LdsLimit seen;
    if (int32_t rc = ensure_lds((const void *)fc_mfma_kernel<NQ>, lds, seen)) return rc;
    dim3 grid;
    GRID_TRY(grid, (int64_t)panels * splits * (np / MfmaShape<NQ>::kImages));
    hipLaunchKernelGGL(fc_mfma_kernel<NQ>, grid, dim3(MfmaShape<NQ>::kThreads), lds, st, D, xt, part, splits, np, panels_per_x, x_stride, out);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

template <int NQ>
int32_t launch_bf16_as(const LayerDev &D, int panels, int splits, int np, int panels_per_x, size_t x_stride, size_t lds,
                       const uint16_t *xb, size_t plane_elems, float *part, hipStream_t st)
{
    static LdsLimit seen;
    if (int32_t rc = ensure_lds((const void *)fc_mfma_bf16_kernel<NQ>, lds, seen)) return rc;
    dim3 grid;
    GRID_TRY(grid, (int64_t)panels * splits * (np / Bf16Shape<NQ>::kImages));
    hipLaunchKernelGGL(fc_mfma_bf16_kernel<NQ>, grid, dim3(Bf16Shape<NQ>::kThreads), lds, st, D, xb, part, splits, np, plane_elems, panels_per_x, x_stride);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

// panels block rows in one launch; each run of panels_per_x of them multiplies an
// activation matrix of its own, x_bytes after the one before
int32_t launch_mfma(const cl_layer *L, const LayerDev &D, bool bf16, int nq, int panels, int splits, int np, int panels_per_x,
                    size_t x_bytes, size_t lds, const void *xt, float *part, hipStream_t st,
                    const DirectOut &out = DirectOut{nullptr, nullptr, 0, 1, 0})
{
    const size_t x_stride = x_bytes / (bf16 ? sizeof(uint16_t) : sizeof(float));
    if (bf16) {
        const size_t pe = xb_plane_elems(L, np);
        switch (nq) {
        case 1: return launch_bf16_as<1>(D, panels, splits, np, panels_per_x, x_stride, lds, (const uint16_t *)xt, pe, part, st);
        case 2: return launch_bf16_as<2>(D, panels, splits, np, panels_per_x, x_stride, lds, (const uint16_t *)xt, pe, part, st);
        case 4: return launch_bf16_as<4>(D, panels, splits, np, panels_per_x, x_stride, lds, (const uint16_t *)xt, pe, part, st);
        case 8: return launch_bf16_as<8>(D, panels, splits, np, panels_per_x, x_stride, lds, (const uint16_t *)xt, pe, part, st);
        }
    } else {
        switch (nq) {
        case 1: return launch_mfma_as<1>(D, panels, splits, np, panels_per_x, x_stride, lds, (const float *)xt, part, out, st);
        case 2: return launch_mfma_as<2>(D, panels, splits, np, panels_per_x, x_stride, lds, (const float *)xt, part, out, st);
        case 4: return launch_mfma_as<4>(D, panels, splits, np, panels_per_x, x_stride, lds, (const float *)xt, part, out, st);
        case 8: return launch_mfma_as<8>(D, panels, splits, np, panels_per_x, x_stride, lds, (const float *)xt, part, out, st);
        }
    }
    return fail(CL_EINVAL, "internal: no dense-tile kernel for %d accumulators", nq);
}

// Launch shape of the wide sparse path (large batches on the vector ALUs).
struct WidePlan {
    int ipl = 4;             // images per lane: the image tile is 64 * ipl images
    int Bp = 0;              // batch rounded up to whole image tiles
    int splits = 1;          // workgroups sharing the blocks of one block row
    int64_t cost = 0;        // modelled cycles of the launches (same units as mfma_shape's)
    size_t lds = 0;
    size_t tile_bytes = 0;   // the partial tiles; behind them in the workspace's partial-tile part:
    size_t ent_bytes = 0;    //   the entry list
    size_t xt_bytes = 0, part_bytes = 0;
};

int32_t plan_wide(const cl_layer *L, int batch, const DeviceLimits &dl, WidePlan &P)
{
    if (!mfma_capable(L)) return fail(CL_EUNSUPPORTED, "the wide sparse path needs blocks of at most %d x %d", kTile, kTile);
    if (batch > kMaxTileColumns) return fail(CL_EUNSUPPORTED, "the wide sparse path takes at most %d images per call", kMaxTileColumns);
    P.ipl = batch > 128 ? 4 : batch > 64 ? 2 : 1;
    const int tile = 64 * P.ipl;
    P.Bp = (batch + tile - 1) / tile * tile;
    // two slabs of 64 columns x tile images, and the codebook
    P.lds = 2 * (size_t)kHalf * tile * sizeof(float) + ((size_t)4 << L->desc.weight_bits);
    if (P.lds > dl.max_lds) return fail(CL_EUNSUPPORTED, "the wide sparse path needs %zu bytes of LDS, %zu there", P.lds, dl.max_lds);
    // Split of the block rows, from a small model of the launches, in cycles per workgroup:
    // a start; per block two phases (one for blocks of at most 64 columns) of 2 k cycles and
    // a part per surviving weight - 9, 6.5 and 5.5 cycles at 4, 2 and 1 images per lane (at 4
    // the LDS port's 8 cycles per KB binds, below it the vector ALUs: 5 and 4 instructions
    // per weight over four SIMDs); the partial tiles, written and read again, as on the
    // dense-tile path; workgroups run in rounds of one per CU; and once per call the
    // decoding launch, 13 k and 6 per thousand entries.  Fitted to the AlexNet-shaped
    // fc6 / fc7 / fc8 at 256 images (multiply 68.7 / 35.1 / 24.8 us, decode 16.2 / 8.5 / 8.0 us).
    const int64_t tiles = (int64_t)L->n_panels * (P.Bp / tile);
    const int cus = std::max(1, dl.cus);
    const int64_t nnz_block = L->n_blocks ? L->nnz / L->n_blocks : 0;
    const int64_t per_weight_x2 = P.ipl == 4 ? 18 : P.ipl == 2 ? 13 : 11;
    const int64_t per_block = (L->desc.block_w > kHalf ? 4000 : 2000) + nnz_block * per_weight_x2 / 2;
    const int64_t start = 12000, once = 13000 + L->entries * 6 / 1000;
    const int sp_max = (int)std::max<int64_t>(1, std::min<int64_t>(L->nbw, (3 * (int64_t)cus + tiles - 1) / tiles));
    int64_t best = -1;
    for (int sp = 1; sp <= sp_max; ++sp) {
        const int64_t rounds = (tiles * sp + cus - 1) / cus, blocks = (L->nbw + sp - 1) / sp;
        const int64_t t = once + rounds * (start + blocks * per_block) +
                          (int64_t)L->n_panels * sp * P.Bp * kTile * (int64_t)sizeof(float) * 3 / 4000;
        if (best < 0 || t < best) {
            best = t;
            P.splits = sp;
        }
    }
    P.cost = best;
    P.xt_bytes = xt_bytes_for(L, P.Bp, false);
    P.tile_bytes = (size_t)L->n_panels * P.splits * kTile * P.Bp * sizeof(float);
    P.ent_bytes = ((size_t)L->nnz * sizeof(WideEntry) + 255) / 256 * 256;
    P.part_bytes = P.tile_bytes + P.ent_bytes;
    return CL_OK;
}

template <int IPL>
int32_t launch_wide_mul(const LayerDev &D, int panels, const WidePlan &P, const float *xt, float *part, const WideEntry *ent,
                        hipStream_t st)
{
    static LdsLimit seen;
    if (int32_t rc = ensure_lds((const void *)wide_mul_kernel<IPL>, P.lds, seen)) return rc;
    dim3 grid;
    GRID_TRY(grid, (int64_t)panels * P.splits * (P.Bp / (64 * IPL)));
    hipLaunchKernelGGL(wide_mul_kernel<IPL>, grid, dim3(kWideThreads), P.lds, st, D, xt, ent, part, panels, P.splits, P.Bp);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

// CL_PATH_AUTO: the sparse path up to kAutoSparseBatch images (one batch tile of the kernel
// with a tile per wavefront); above, when the blocks fit a tile, whichever of the dense-tile
// path and the wide sparse path the two launch models price lower (same units, both fitted
// to measured launches).  Measured on the AlexNet-shaped stack (fc6 / fc7 / fc8, ms per
// layer call): sparse 0.019 / 0.015 / 0.015 at 4 images, 0.024 / 0.016 / 0.014 at 8 and
// 0.054 / 0.034 / 0.024 at 9-16 (two batch tiles); dense tiles of 32 images 0.040 / 0.024 /
// 0.019; at 256 images dense tiles 0.176 / 0.095 / 0.044, wide sparse 0.094 / 0.051 for fc6
// and fc7 - the dense tile multiplies eleven times the necessary products at a 9 % density
// but four at 25 %.
constexpr int kAutoSparseBatch = 8;

int resolve_path(const cl_layer *L, int batch, int path, const DeviceLimits &dl)
{
    if (path != CL_PATH_AUTO) return path;
    if (batch <= kAutoSparseBatch || !mfma_capable(L)) return CL_PATH_SPARSE;
    if (batch > kMaxTileColumns) return CL_PATH_MFMA_F32;      // refused there with its message
    WidePlan W;
    if (plan_wide(L, batch, dl, W) != CL_OK) {
        clear_error();
        return CL_PATH_MFMA_F32;
    }
    int nq, np, splits;
    int64_t dense = 0;
    mfma_shape(L, L->n_panels, batch, dl.cus, false, nq, np, splits, false, false, &dense);
    return W.cost < dense ? CL_PATH_SPARSE_WIDE : CL_PATH_MFMA_F32;
}

bool is_mfma(int path) { return path == CL_PATH_MFMA_F32 || path == CL_PATH_MFMA_BF16; }

// the paths that read the activations transposed and laid out block by block
bool reads_xt(int path) { return is_mfma(path) || path == CL_PATH_SPARSE_WIDE; }

}  // namespace

extern "C" int32_t cl_fc_workspace_bytes(const cl_layer *L, int32_t batch, int32_t path, size_t *out)
{
    if (!L || !out) return fail(CL_EINVAL, "null argument");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    if (path < CL_PATH_AUTO || path > CL_PATH_SPARSE_WIDE) return fail(CL_EINVAL, "unknown path %d", path);
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    const int chosen = resolve_path(L, batch, path, dl);
    if (chosen == CL_PATH_SPARSE_WIDE) {
        WidePlan P;
        if (int32_t rc = plan_wide(L, batch, dl, P)) return rc;
        *out = P.xt_bytes + P.part_bytes;
    } else if (is_mfma(chosen)) {
        MfmaPlan P;
        if (int32_t rc = plan_mfma(L, batch, chosen == CL_PATH_MFMA_BF16, dl, P)) return rc;
        *out = P.xt_bytes + P.part_bytes;
    } else {
        SparsePlan P;
        if (int32_t rc = plan_sparse(L, batch, dl.max_lds, P)) return rc;
        *out = P.part_bytes;
    }
    return CL_OK;
}

extern "C" int32_t cl_fc_resolved_path(const cl_layer *L, int32_t batch, int32_t path, int32_t *out)
{
    if (!L || !out) return fail(CL_EINVAL, "null argument");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    if (path < CL_PATH_AUTO || path > CL_PATH_SPARSE_WIDE) return fail(CL_EINVAL, "unknown path %d", path);
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    *out = resolve_path(L, batch, path, dl);
    return CL_OK;
}

// The small-batch path for one layer.  With `prev` the input is not d_X but the partial
// tiles of the layer before (see PrevSlots); with finish == false the layer's own
// finishing kernel is left to the layer after it in the same way.  Both only where
// sparse_can_fold allows.
static int32_t forward_sparse(const cl_layer *L, const LayerDev &D, const DeviceLimits &dl, const float *d_X,
                              const float *d_bias, float *d_Y, int batch, int relu, float *part, hipStream_t st,
                              const PrevSlots *prev = nullptr, bool finish = true)
{
    SparsePlan P;
    if (int32_t rc = plan_sparse(L, batch, dl.max_lds, P)) return rc;
    const PrevSlots from = prev ? *prev : PrevSlots{nullptr, nullptr, nullptr, 1, 0, 0, 0};
    if ((prev || !finish) && !sparse_can_fold(L, P, batch)) return fail(CL_EINVAL, "internal: layer cannot take or leave partial tiles");
    const int M = L->desc.M, K = L->desc.K;
    dim3 grid;
    if (L->n_chunks > 0) GRID_TRY(grid, (int64_t)L->n_panels * P.wg_per_panel);
    for (int b0 = 0; b0 < batch;) {
        // the smallest batch tile that holds the images left (its other images are zeros):
        // one launch for 3 images, not two
        const int nb = std::min(P.bt_max, batch - b0);
        int bt = P.bt_max;
        while (bt / 2 >= nb) bt >>= 1;
        const float *x = d_X + (size_t)b0 * K;
        float *y = d_Y + (size_t)b0 * M;
        if (L->n_chunks > 0) {
            const size_t lds = P.lds_for(L, bt);
            const int xcap = P.xcap_for(bt);
            if (b0 == 0) timing_begin(st);      // benchmarks time the first main-kernel launch of a call
#define CL_LAUNCH_SPARSE(BTV, FOLDV)                                                                               \
    do {                                                                                                           \
        if (lds > 64 * 1024)                                                                                       \
            HIP_TRY(hipFuncSetAttribute((const void *)fc_sparse_kernel<BTV, FOLDV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
        hipLaunchKernelGGL((fc_sparse_kernel<BTV, FOLDV>), grid, dim3(kThreads), lds, st, D, x, part, P.wg_per_panel, xcap, from, nb); \
    } while (0)
            switch (bt) {
            case 16: CL_LAUNCH_SPARSE(16, false); break;
            case 8: CL_LAUNCH_SPARSE(8, false); break;
            case 4: CL_LAUNCH_SPARSE(4, false); break;
            case 2: CL_LAUNCH_SPARSE(2, false); break;
            default:
                if (prev) CL_LAUNCH_SPARSE(1, true);
                else CL_LAUNCH_SPARSE(1, false);
                break;
            }
#undef CL_LAUNCH_SPARSE
            HIP_TRY(hipGetLastError());
            if (b0 == 0) timing_end(st, 1);
        }
        if (finish) {
            dim3 rgrid;
            GRID_TRY(rgrid, (int64_t)L->n_panels * nb);
            hipLaunchKernelGGL(fc_reduce_kernel, rgrid, dim3(kRedThreads), 0, st,
                               D, part, d_bias, y, nb, bt, P.wg_per_panel, relu);
            HIP_TRY(hipGetLastError());
        }
        b0 += nb;
    }
    return CL_OK;
}

// One layer on a dense-tile path with launch shape P.  The input is d_X (batch x K, laid
// out for the kernel into xt first) or, when d_X is null, already sits in xt.  The
// output goes to d_Y as batch x M, or, with next_bp > 0, as the transposed activations
// of a following 128-column-block layer whose image axis is padded to next_bp
// (Y[row][next_bp], padded images zero).
static int32_t run_mfma_layer(const cl_layer *L, const LayerDev &D, const MfmaPlan &P, const float *d_X, void *xt, float *part,
                              const float *d_bias, float *d_Y, int next_bp, int batch, int relu, hipStream_t st)
{
    const int K = L->desc.K;
    if (d_X) {
        if (P.bf16) {
            hipLaunchKernelGGL(split_pad_kernel, dim3((unsigned)(L->nbw * 8), (unsigned)((P.Bp + 63) / 64)), dim3(256), 0, st,
                               d_X, (uint16_t *)xt, batch, K, P.Bp, L->desc.block_w, xb_plane_elems(L, P.Bp));
        } else {
            const int rows = L->nbw * kTile;
            hipLaunchKernelGGL(transpose_pad_kernel, dim3((unsigned)(rows / 32), (unsigned)(P.Bp / 32)), dim3(256), 0, st,
                               d_X, (float *)xt, batch, K, P.Bp, L->desc.block_w, rows);
        }
        HIP_TRY(hipGetLastError());
    }
    timing_begin(st);
    if (int32_t rc = launch_mfma(L, D, P.bf16, P.nq, L->n_panels, P.splits, P.Bp, L->n_panels, 0, P.lds, xt, part, st)) return rc;
    timing_end(st, 1);
    const int cols = std::max(batch, next_bp);
    // towards a following layer the output runs along the images: full 32-column tiles
    // (128-byte runs), and the rows of a block row shared out to keep the launch wide
    int ct = reduce_col_tile(L->n_panels, cols), rt = L->desc.block_h;
    if (next_bp > 0) {
        ct = kColTile;
        rt = kTile;
        while (rt > 32 && (int64_t)L->n_panels * ((cols + ct - 1) / ct) * ((L->desc.block_h + rt - 1) / rt) < 1024) rt >>= 1;
    }
    const int nrt = (L->desc.block_h + rt - 1) / rt;
    dim3 rgrid;
    GRID_TRY(rgrid, (int64_t)L->n_panels * ((cols + ct - 1) / ct) * nrt);
    hipLaunchKernelGGL(mfma_reduce_kernel, rgrid, dim3(256), 0, st,
                       D, part, d_bias, d_Y, batch, P.Bp, P.splits, relu, next_bp, ct, next_bp, rt);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

// The decoding launch of the wide path for up to kExpandJobs layers at once, each
// into its own list.  Layers without chunks are skipped (their lists are empty).
// (xt_of: the layer whose activations d_X, batch x K, the launch lays out as well, into xt
// with the image axis padded to bp - or null)
static int32_t launch_wide_expand(const cl_layer *const *layers, WideEntry *const *ents, int n, int ipl, hipStream_t st,
                                  const cl_layer *xt_of = nullptr, const float *d_X = nullptr, float *xt = nullptr, int batch = 0,
                                  int bp = 0)
{
    ExpandJobs jobs{};
    jobs.ipl = (uint32_t)ipl;
    size_t lds = 0;
    int64_t wgs = 0;
    int used = 0;
    if (xt_of) {
        jobs.X = d_X;
        jobs.XT = xt;
        jobs.B = batch;
        jobs.K = xt_of->desc.K;
        jobs.Bp = bp;
        jobs.bw = xt_of->desc.block_w;
        jobs.rows = xt_of->nbw * kTile;
        jobs.t_wgs = (uint32_t)(((int64_t)(jobs.rows / 32) * (bp / 32) + 1) / 2);
        wgs = jobs.t_wgs;
    }
    for (int i = 0; i < n; ++i) {
        const cl_layer *L = layers[i];
        if (L->n_chunks == 0) continue;
        jobs.L[used] = make_dev(L);
        jobs.ent[used] = ents[i];
        jobs.wg0[used] = (uint32_t)wgs;
        wgs += (L->n_chunks + kWaves - 1) / kWaves;
        lds = std::max(lds, table_image_bytes(L->val_lut_bits, L->idx_lut_bits, 1 << L->desc.weight_bits));
        ++used;
    }
    if (!used && !jobs.t_wgs) return CL_OK;
    for (int i = used; i <= kExpandJobs; ++i) jobs.wg0[i] = i == used ? (uint32_t)wgs : UINT32_MAX;
    if (!used) {
        // nothing to decode: the launch only lays the activations out (the job table names the
        // first layer, whose range of workgroups is empty)
        jobs.L[0] = make_dev(xt_of);
        jobs.wg0[0] = (uint32_t)wgs;
    }
    for (int i = std::max(used, 1); i < kExpandJobs; ++i) jobs.L[i] = jobs.L[0];
    static LdsLimit seen;
    if (int32_t rc = ensure_lds((const void *)wide_expand_kernel, lds, seen)) return rc;
    dim3 egrid;
    GRID_TRY(egrid, wgs);
    hipLaunchKernelGGL(wide_expand_kernel, egrid, dim3(kThreads), lds, st, jobs);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

// One layer on the wide sparse path with launch shape P; arguments as run_mfma_layer.  The
// entry list is `ent`; with expanded it has been written already (by a launch_wide_expand
// that took several layers of a stack together).
static int32_t run_wide_layer(const cl_layer *L, const LayerDev &D, const WidePlan &P, const float *d_X, float *xt, float *part,
                              WideEntry *ent, bool expanded, const float *d_bias, float *d_Y, int next_bp, int batch, int relu,
                              hipStream_t st)
{
    int32_t rc = CL_EINVAL;
    if (!expanded) {
        // one launch decodes the layer and lays its activations out
        if ((rc = launch_wide_expand(&L, &ent, 1, P.ipl, st, d_X ? L : nullptr, d_X, xt, batch, P.Bp))) return rc;
    } else if (d_X) {
        const int rows = L->nbw * kTile;
        hipLaunchKernelGGL(transpose_pad_kernel, dim3((unsigned)(rows / 32), (unsigned)(P.Bp / 32)), dim3(256), 0, st,
                           d_X, xt, batch, L->desc.K, P.Bp, L->desc.block_w, rows);
        HIP_TRY(hipGetLastError());
    }
    timing_begin(st);
    switch (P.ipl) {
    case 1: rc = launch_wide_mul<1>(D, L->n_panels, P, xt, part, ent, st); break;
    case 2: rc = launch_wide_mul<2>(D, L->n_panels, P, xt, part, ent, st); break;
    case 4: rc = launch_wide_mul<4>(D, L->n_panels, P, xt, part, ent, st); break;
    }
    if (rc) return rc;
    timing_end(st, 1);
    const int ncol = std::max(P.Bp, next_bp);
    dim3 rgrid;
    GRID_TRY(rgrid, (int64_t)L->n_panels * (kTile / kWideRedRows) * ((ncol + kWideRedImages - 1) / kWideRedImages));
    hipLaunchKernelGGL(wide_reduce_kernel, rgrid, dim3(256), 0, st, D, part, d_bias, d_Y, batch, P.Bp, P.splits, relu, next_bp);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

static int32_t forward_wide(const cl_layer *L, const LayerDev &D, const DeviceLimits &dl, const float *d_X, const float *d_bias,
                            float *d_Y, int batch, int relu, char *ws, hipStream_t st)
{
    WidePlan P;
    if (int32_t rc = plan_wide(L, batch, dl, P)) return rc;
    return run_wide_layer(L, D, P, d_X, (float *)ws, (float *)(ws + P.xt_bytes), (WideEntry *)(ws + P.xt_bytes + P.tile_bytes), false,
                          d_bias, d_Y, 0, batch, relu, st);
}

static int32_t forward_mfma(const cl_layer *L, const LayerDev &D, const DeviceLimits &dl, bool bf16, const float *d_X,
                            const float *d_bias, float *d_Y, int batch, int relu, char *ws, hipStream_t st)
{
    MfmaPlan P;
    if (int32_t rc = plan_mfma(L, batch, bf16, dl, P)) return rc;
    return run_mfma_layer(L, D, P, d_X, ws, (float *)(ws + P.xt_bytes), d_bias, d_Y, 0, batch, relu, st);
}

static int32_t fc_forward_checked(const cl_layer *L, const float *d_X, const float *d_bias, float *d_Y, int32_t batch,
                                  int32_t relu, int32_t path, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (int32_t rc = require_device(L)) return rc;
    if (!d_X || !d_Y) return fail(CL_EINVAL, "null activation pointer");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    size_t need = 0;
    if (int32_t rc = cl_fc_workspace_bytes(L, batch, path, &need)) return rc;
    if (workspace_bytes < need || (need && !d_workspace)) return fail(CL_EINVAL, "workspace too small: %zu < %zu", workspace_bytes, need);
    if ((uintptr_t)d_workspace % 256) return fail(CL_EINVAL, "workspace must be 256-byte aligned");
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    const LayerDev D = make_dev(L);
    int32_t rc;
    const int chosen = resolve_path(L, batch, path, dl);
    if (chosen == CL_PATH_SPARSE_WIDE)
        rc = forward_wide(L, D, dl, d_X, d_bias, d_Y, batch, relu, (char *)d_workspace, (hipStream_t)stream);
    else if (is_mfma(chosen))
        rc = forward_mfma(L, D, dl, chosen == CL_PATH_MFMA_BF16, d_X, d_bias, d_Y, batch, relu, (char *)d_workspace, (hipStream_t)stream);
    else
        rc = forward_sparse(L, D, dl, d_X, d_bias, d_Y, batch, relu, (float *)d_workspace, (hipStream_t)stream);
    if (rc == CL_OK) clear_error();
    return rc;
}

extern "C" int32_t cl_compressed_fc_forward(const cl_layer *L, const float *d_X, const float *d_bias,
                                            float *d_Y, int32_t batch, int32_t relu, int32_t path,
                                            void *d_workspace, size_t workspace_bytes, void *stream)
{
    return fc_forward_checked(L, d_X, d_bias, d_Y, batch, relu, path, d_workspace, workspace_bytes, stream);
}

extern "C" int32_t cl_compressed_fc_forward_static(const cl_layer *L, const float *d_X, const float *d_bias,
                                                   float *d_Y, int32_t batch, int32_t relu, int32_t path, void *stream)
{
    if (int32_t rc = require_device(L)) return rc;
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    size_t need = 0;
    if (int32_t rc = cl_fc_workspace_bytes(L, batch, path, &need)) return rc;
    if (need > (size_t)CL_STATIC_SCRATCH_BYTES)
        return fail(CL_EUNSUPPORTED, "this call needs %zu bytes of scratch, the static scratch area holds %zu: use cl_compressed_fc_forward with a workspace",
                    need, (size_t)CL_STATIC_SCRATCH_BYTES);
    void *scratch = nullptr;
    if (int32_t rc = static_scratch(&scratch)) return rc;
    return fc_forward_checked(L, d_X, d_bias, d_Y, batch, relu, path, scratch, (size_t)CL_STATIC_SCRATCH_BYTES, stream);
}

// ------------------------------------------------------------------------- //
// a stack of fully connected layers (Eq. 1 layer after layer)
// ------------------------------------------------------------------------- //
namespace {

struct StackPlan {
    std::vector<int> path;            // per layer: the path it runs on
    std::vector<MfmaPlan> mfma;       // per layer on a dense-tile path
    std::vector<WidePlan> wide;       // per layer on the wide sparse path
    std::vector<SparsePlan> sparse;   // per layer on the sparse path
    std::vector<char> xt_in;          // layer reads its transposed activations straight from the layer before
    std::vector<char> fold_in;        // layer adds up the partial tiles of the layer before itself (both on the sparse path)
    std::vector<size_t> ent_off;      // per layer on the wide path: its entry list in the area behind the rotating buffers
    size_t xt_bytes = 0, part_bytes = 0, act_bytes = 0, ent_bytes = 0;
    int regions = 1;                  // copies of each buffer, used in rotation
    size_t total() const { return (size_t)regions * (xt_bytes + part_bytes + act_bytes) + ent_bytes; }
};

size_t round256(size_t n) { return (n + 255) / 256 * 256; }

constexpr int kStackRegions = 4;

int32_t plan_stack(const cl_layer *const *layers, int n, int batch, int path, const DeviceLimits &dl, StackPlan &P)
{
    if (!layers || n < 1) return fail(CL_EINVAL, "a stack needs at least one layer");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    if (path < CL_PATH_AUTO || path > CL_PATH_SPARSE_WIDE) return fail(CL_EINVAL, "unknown path %d", path);
    P.path.assign(n, 0);
    P.wide.assign(n, WidePlan{});
    P.mfma.assign(n, MfmaPlan{});
    P.sparse.assign(n, SparsePlan{});
    P.xt_in.assign(n, 0);
    P.fold_in.assign(n, 0);
    P.ent_off.assign(n, 0);
    for (int i = 0; i < n; ++i) {
        const cl_layer *L = layers[i];
        if (!L) return fail(CL_EINVAL, "layer %d is null", i);
        if (i > 0 && L->desc.K != layers[i - 1]->desc.M)
            return fail(CL_EINVAL, "layer %d takes %d inputs, layer %d gives %d outputs", i, L->desc.K, i - 1, layers[i - 1]->desc.M);
        P.path[i] = resolve_path(L, batch, path, dl);
        // the finishing kernel of the layer before can write this layer's transposed
        // activations itself when their row order is the plain one (128-column blocks,
        // no ragged last block): 2-3 % of a step on the AlexNet-shaped stack
        const bool plain_rows = L->desc.block_w == kTile && L->desc.K % kTile == 0;
        if (P.path[i] == CL_PATH_SPARSE_WIDE) {
            if (int32_t rc = plan_wide(L, batch, dl, P.wide[i])) return rc;
            P.xt_bytes = std::max(P.xt_bytes, P.wide[i].xt_bytes);
            P.part_bytes = std::max(P.part_bytes, round256(P.wide[i].tile_bytes));
            P.ent_off[i] = P.ent_bytes;
            P.ent_bytes += round256(P.wide[i].ent_bytes);
            P.xt_in[i] = i > 0 && reads_xt(P.path[i - 1]) && plain_rows;
        } else if (is_mfma(P.path[i])) {
            if (int32_t rc = plan_mfma(L, batch, P.path[i] == CL_PATH_MFMA_BF16, dl, P.mfma[i])) return rc;
            P.xt_bytes = std::max(P.xt_bytes, P.mfma[i].xt_bytes);
            P.part_bytes = std::max(P.part_bytes, round256(P.mfma[i].part_bytes));
            P.xt_in[i] = i > 0 && reads_xt(P.path[i - 1]) && P.path[i] == CL_PATH_MFMA_F32 && plain_rows;
        } else {
            if (int32_t rc = plan_sparse(L, batch, dl.max_lds, P.sparse[i])) return rc;
            P.part_bytes = std::max(P.part_bytes, round256(P.sparse[i].part_bytes));
            // (measured on the AlexNet-shaped stack: 39.8 -> 37.1 us at one image, no gain at
            // two, a loss at four - every workgroup of a block column adds the same tiles up)
            P.fold_in[i] = batch == 1 && i > 0 && P.path[i - 1] == CL_PATH_SPARSE && sparse_can_fold(layers[i - 1], P.sparse[i - 1], batch) &&
                           sparse_can_fold(L, P.sparse[i], batch);
        }
        if (i + 1 < n) P.act_bytes = std::max(P.act_bytes, round256((size_t)batch * L->desc.M * sizeof(float)));
    }
    P.regions = std::min(n, kStackRegions);
    return CL_OK;
}

}  // namespace

extern "C" int32_t cl_fc_stack_workspace_bytes(const cl_layer *const *layers, int32_t n_layers, int32_t batch, int32_t path,
                                               size_t *out)
{
    if (!out) return fail(CL_EINVAL, "null argument");
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    StackPlan P;
    if (int32_t rc = plan_stack(layers, n_layers, batch, path, dl, P)) return rc;
    *out = P.total();
    return CL_OK;
}

extern "C" int32_t cl_compressed_fc_stack_forward(const cl_layer *const *layers, int32_t n_layers, const float *d_X,
                                                  const float *const *d_bias_or_null, float *d_Y, int32_t batch,
                                                  int32_t relu_hidden, int32_t relu_last, int32_t path, void *d_workspace,
                                                  size_t workspace_bytes, void *stream)
{
    if (!d_X || !d_Y) return fail(CL_EINVAL, "null activation pointer");
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    StackPlan P;
    if (int32_t rc = plan_stack(layers, n_layers, batch, path, dl, P)) return rc;
    for (int i = 0; i < n_layers; ++i)
        if (int32_t rc = require_device(layers[i])) return rc;
    if (workspace_bytes < P.total() || (P.total() && !d_workspace))
        return fail(CL_EINVAL, "workspace too small: %zu < %zu", workspace_bytes, P.total());
    if ((uintptr_t)d_workspace % 256) return fail(CL_EINVAL, "workspace must be 256-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)d_workspace;
    // Up to four of everything, used in rotation.  Two would do for the data's lifetime;
    // more are a matter of speed: a kernel that writes where a kernel shortly before has
    // read (the partial tiles above all) runs slower, the lines being still held by the
    // other dies' caches - 3 % of a step at batch 256 with one buffer of partial tiles,
    // 5 % at batch 64 with two.
    const int R = P.regions;
    auto region = [&](size_t base, size_t bytes, int i) { return ws + base + (size_t)(i % R) * bytes; };
    const size_t xt0 = 0, part0 = (size_t)R * P.xt_bytes, act0 = part0 + (size_t)R * P.part_bytes;
    // The layers on the wide path are decoded up front, kExpandJobs to a launch: the
    // lists depend on the weights only, and one launch for two layers is shorter than two
    // (the fixed part of such a launch - start, tables, the dependent loads - is a third of fc7's).
    const size_t ent0 = act0 + (size_t)R * P.act_bytes;
    auto ent_of = [&](int i) { return (WideEntry *)(ws + ent0 + P.ent_off[i]); };
    // (the first of these launches also lays out the input of the stack when its first layer is
    // one of them)
    bool x_laid_out = false;
    {
        const cl_layer *todo[kExpandJobs];
        WideEntry *ents[kExpandJobs];
        int n = 0, ipl_of_stack = 4;                 // (the images per lane follow from the batch: the same for every layer)
        for (int i = 0; i <= n_layers; ++i) {
            const bool mine = i < n_layers && P.path[i] == CL_PATH_SPARSE_WIDE;
            if (mine) {
                todo[n] = layers[i];
                ents[n] = ent_of(i);
                ipl_of_stack = P.wide[i].ipl;
                ++n;
            }
            if (n == kExpandJobs || (i == n_layers && n > 0)) {
                const bool with_x = !x_laid_out && P.path[0] == CL_PATH_SPARSE_WIDE;
                if (int32_t rc = launch_wide_expand(todo, ents, n, ipl_of_stack, st, with_x ? layers[0] : nullptr, d_X,
                                                    (float *)region(xt0, P.xt_bytes, 0), batch, P.wide[0].Bp))
                    return rc;
                x_laid_out = x_laid_out || with_x;
                n = 0;
            }
        }
    }
    const float *in = x_laid_out ? nullptr : d_X;    // the layer's input as batch x K, or null when it sits in its xt region
    for (int i = 0; i < n_layers; ++i) {
        const cl_layer *L = layers[i];
        const LayerDev D = make_dev(L);
        const bool last = i + 1 == n_layers;
        const float *bias = d_bias_or_null ? d_bias_or_null[i] : nullptr;
        const int relu = last ? relu_last : relu_hidden;
        float *out = last ? d_Y : (float *)region(act0, P.act_bytes, i);
        if (reads_xt(P.path[i])) {
            // towards a following layer that takes its activations transposed, this layer's finishing
            // kernel writes them so, the image axis padded to that layer's tile
            const bool to_xt = !last && P.xt_in[i + 1];
            float *dst = to_xt ? (float *)region(xt0, P.xt_bytes, i + 1) : out;
            const int next_bp = !to_xt ? 0 : P.path[i + 1] == CL_PATH_SPARSE_WIDE ? P.wide[i + 1].Bp : P.mfma[i + 1].Bp;
            int32_t rc;
            if (P.path[i] == CL_PATH_SPARSE_WIDE)
                rc = run_wide_layer(L, D, P.wide[i], in, (float *)region(xt0, P.xt_bytes, i), (float *)region(part0, P.part_bytes, i),
                                    ent_of(i), true, bias, dst, next_bp, batch, relu, st);
            else
                rc = run_mfma_layer(L, D, P.mfma[i], in, region(xt0, P.xt_bytes, i), (float *)region(part0, P.part_bytes, i), bias, dst, next_bp, batch, relu, st);
            if (rc) return rc;
            in = to_xt ? nullptr : out;
        } else {
            // between two layers of this path at one image the finishing kernel is left out:
            // the next layer adds the partial tiles up as it stages its input
            PrevSlots prev{};
            if (P.fold_in[i]) {
                const cl_layer *Lp = layers[i - 1];
                prev = PrevSlots{(const float *)region(part0, P.part_bytes, i - 1), make_dev(Lp).panel_chunk,
                                 d_bias_or_null ? d_bias_or_null[i - 1] : nullptr, Lp->desc.block_h, P.sparse[i - 1].wg_per_panel,
                                 batch, relu_hidden};
            }
            const bool finish = last || !P.fold_in[i + 1];
            if (int32_t rc = forward_sparse(L, D, dl, in, bias, out, batch, relu, (float *)region(part0, P.part_bytes, i), st,
                                            P.fold_in[i] ? &prev : nullptr, finish))
                return rc;
            in = out;
        }
    }
    clear_error();
    return CL_OK;
}

// ------------------------------------------------------------------------- //
// several layers of one shape in one grid
// ------------------------------------------------------------------------- //
struct cl_layer_group {
    std::vector<const cl_layer *> layers;
    LayerDev *table = nullptr;        // device copy of the layers' LayerDev, in order
    int device = -1;
    int64_t max_panel_chunks = 0;     // over all layers
    size_t table_bytes = 0;           // largest table image (LDS) of any layer
    bool any_chunks = false;
};

namespace {

struct GroupPlan {
    SparsePlan sp;
    uint32_t wgs_per_layer = 0;
    size_t part_stride = 0;           // floats between the layers' partial tiles
    size_t lds = 0;
    int xcap = 0;
};

int32_t plan_group(const cl_layer_group *G, int batch, const DeviceLimits &dl, GroupPlan &P)
{
    const cl_layer *L = G->layers[0];
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    if (batch > 16 || (batch & (batch - 1))) return fail(CL_EUNSUPPORTED, "a group call takes 1, 2, 4, 8 or 16 images per layer");
    if (int32_t rc = plan_sparse(L, batch, dl.max_lds, P.sp, true)) return rc;
    if (P.sp.bt_max < batch) return fail(CL_EUNSUPPORTED, "%d images do not fit one batch tile of this layer shape", batch);
    const int bt = batch;
    P.sp.bt_max = bt;
    P.sp.fixed = G->table_bytes;
    P.sp.wg_per_panel = (int)((G->max_panel_chunks + kWaves * kSparseChunksPerWave - 1) / (kWaves * kSparseChunksPerWave));
    P.wgs_per_layer = (uint32_t)std::max<int64_t>(1, (int64_t)L->n_panels * P.sp.wg_per_panel);
    P.part_stride = (size_t)P.wgs_per_layer * L->desc.block_h * bt;
    P.lds = P.sp.lds_for(L, bt);
    if (P.lds > dl.max_lds) return fail(CL_EUNSUPPORTED, "the layers' tables and a tile of %d images need more LDS than a workgroup has", bt);
    P.xcap = P.sp.xcap_for(bt);
    return CL_OK;
}

}  // namespace

extern "C" int32_t cl_layer_group_create(const cl_layer *const *layers, int32_t n_layers, cl_layer_group **out)
{
    if (!layers || !out || n_layers < 1) return fail(CL_EINVAL, "a group needs at least one layer");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    std::unique_ptr<cl_layer_group> G(new cl_layer_group());
    std::vector<LayerDev> host;
    for (int i = 0; i < n_layers; ++i) {
        const cl_layer *L = layers[i];
        if (int32_t rc = require_device(L)) return rc;
        const cl_layer *F = layers[0];
        if (L->desc.M != F->desc.M || L->desc.K != F->desc.K || L->desc.block_h != F->desc.block_h || L->desc.block_w != F->desc.block_w)
            return fail(CL_EINVAL, "layer %d differs from layer 0 in shape or block size", i);
        G->layers.push_back(L);
        host.push_back(make_dev(L));
        G->max_panel_chunks = std::max(G->max_panel_chunks, L->max_panel_chunks);
        G->table_bytes = std::max(G->table_bytes, table_image_bytes(L->val_lut_bits, L->idx_lut_bits, 1 << L->desc.weight_bits));
        G->any_chunks = G->any_chunks || L->n_chunks > 0;
    }
    G->device = dev;
    if (hipMalloc((void **)&G->table, host.size() * sizeof(LayerDev)) != hipSuccess)
        return fail(CL_ENOMEM, "hipMalloc of the group table failed");
    if (hipMemcpy(G->table, host.data(), host.size() * sizeof(LayerDev), hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(G->table);
        return fail(CL_EHIP, "hipMemcpy of the group table failed");
    }
    *out = G.release();
    clear_error();
    return CL_OK;
}

extern "C" void cl_layer_group_free(cl_layer_group *G)
{
    if (!G) return;
    if (G->table) (void)hipFree(G->table);
    delete G;
}

extern "C" int32_t cl_fc_group_workspace_bytes(const cl_layer_group *G, int32_t batch, size_t *out)
{
    if (!G || !out) return fail(CL_EINVAL, "null argument");
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    GroupPlan P;
    if (int32_t rc = plan_group(G, batch, dl, P)) return rc;
    *out = G->layers.size() * P.part_stride * sizeof(float);
    return CL_OK;
}

extern "C" int32_t cl_compressed_fc_group_forward(const cl_layer_group *G, const float *d_X, size_t x_stride,
                                                  const float *d_bias_or_null, size_t bias_stride, float *d_Y, int32_t batch,
                                                  int32_t relu, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!G || !d_X || !d_Y) return fail(CL_EINVAL, "null argument");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != G->device) return fail(CL_EINVAL, "the group was created on device %d, the current device is %d", G->device, dev);
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    GroupPlan P;
    if (int32_t rc = plan_group(G, batch, dl, P)) return rc;
    const size_t n = G->layers.size(), need = n * P.part_stride * sizeof(float);
    if (workspace_bytes < need || !d_workspace) return fail(CL_EINVAL, "workspace too small: %zu < %zu", workspace_bytes, need);
    if ((uintptr_t)d_workspace % 256) return fail(CL_EINVAL, "workspace must be 256-byte aligned");
    const cl_layer *L = G->layers[0];
    hipStream_t st = (hipStream_t)stream;
    float *part = (float *)d_workspace;
    const int bt = P.sp.bt_max;
    if (G->any_chunks) {
        dim3 grid;
        GRID_TRY(grid, (int64_t)n * P.wgs_per_layer);
        timing_begin(st);
#define CL_LAUNCH_GROUP(BTV)                                                                                        \
    do {                                                                                                            \
        if (P.lds > 64 * 1024)                                                                                      \
            HIP_TRY(hipFuncSetAttribute((const void *)fc_sparse_group_kernel<BTV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)P.lds)); \
        hipLaunchKernelGGL(fc_sparse_group_kernel<BTV>, grid, dim3(kThreads), P.lds, st, G->table, P.wgs_per_layer, d_X, x_stride, part, \
                           P.part_stride, P.sp.wg_per_panel, P.xcap);                                               \
    } while (0)
        switch (bt) {
        case 16: CL_LAUNCH_GROUP(16); break;
        case 8: CL_LAUNCH_GROUP(8); break;
        case 4: CL_LAUNCH_GROUP(4); break;
        case 2: CL_LAUNCH_GROUP(2); break;
        default: CL_LAUNCH_GROUP(1); break;
        }
#undef CL_LAUNCH_GROUP
        HIP_TRY(hipGetLastError());
        timing_end(st, 1);
    }
    const int red_per_layer = L->n_panels * bt;
    dim3 rgrid;
    GRID_TRY(rgrid, (int64_t)n * red_per_layer);
    hipLaunchKernelGGL(fc_reduce_group_kernel, rgrid, dim3(kRedThreads), 0, st, G->table, red_per_layer, part, P.part_stride,
                       d_bias_or_null, bias_stride, d_Y, (size_t)batch * L->desc.M, bt, P.sp.wg_per_panel, relu);
    HIP_TRY(hipGetLastError());
    clear_error();
    return CL_OK;
}

// ------------------------------------------------------------------------- //
// fixed-function layers of a whole network (Table IV: pool, norm)
// ------------------------------------------------------------------------- //

extern "C" int32_t cl_maxpool_forward(const float *d_X, float *d_Y, int32_t batch, int32_t C, int32_t H, int32_t W,
                                      int32_t size, int32_t stride, void *stream)
{
    if (!d_X || !d_Y) return fail(CL_EINVAL, "null pointer");
    if (batch < 1 || C < 1 || size < 1 || stride < 1 || H < size || W < size) return fail(CL_EINVAL, "bad pooling geometry");
    const int P = (H - size) / stride + 1, Q = (W - size) / stride + 1;
    if ((int64_t)P * Q > (1 << 30)) return fail(CL_EUNSUPPORTED, "more than 2^30 outputs per plane");
    const int64_t planes = (int64_t)batch * C;
    const int pq = P * Q, planes_per_row = (int)std::min<int64_t>(planes, std::max(1, 2048 / pq));
    const dim3 grid((unsigned)(((int64_t)planes_per_row * pq + 255) / 256),
                    (unsigned)std::min<int64_t>((planes + planes_per_row - 1) / planes_per_row, 65535));
    auto kernel = size == 3 ? maxpool_kernel<3> : size == 2 ? maxpool_kernel<2> : maxpool_kernel<0>;
    hipLaunchKernelGGL(kernel, grid, dim3(256), 0, (hipStream_t)stream, d_X, d_Y, planes, H, W, P, Q, size, stride, planes_per_row);
    HIP_TRY(hipGetLastError());
    clear_error();
    return CL_OK;
}

extern "C" int32_t cl_lrn_forward(const float *d_X, float *d_Y, int32_t batch, int32_t C, int32_t H, int32_t W,
                                  int32_t n, float alpha, float beta, float k, void *stream)
{
    if (!d_X || !d_Y) return fail(CL_EINVAL, "null pointer");
    if (batch < 1 || C < 1 || H < 1 || W < 1 || n < 1 || !(n & 1)) return fail(CL_EINVAL, "bad normalisation geometry");
    const int64_t hw = (int64_t)H * W, runs = (int64_t)batch * ((C + kLrnChunk - 1) / kLrnChunk);
    if (runs > INT32_MAX) return fail(CL_EUNSUPPORTED, "batch x channels too large");
    const dim3 grid((unsigned)((hw + 255) / 256), (unsigned)std::min<int64_t>(runs, 65535));
    const float a_n = alpha / (float)n;
    switch (n / 2) {
    case 1: hipLaunchKernelGGL(lrn_kernel<1>, grid, dim3(256), 0, (hipStream_t)stream, d_X, d_Y, batch, C, hw, n, a_n, beta, k); break;
    case 2: hipLaunchKernelGGL(lrn_kernel<2>, grid, dim3(256), 0, (hipStream_t)stream, d_X, d_Y, batch, C, hw, n, a_n, beta, k); break;
    default: hipLaunchKernelGGL(lrn_kernel<-1>, grid, dim3(256), 0, (hipStream_t)stream, d_X, d_Y, batch, C, hw, n, a_n, beta, k); break;
    }
    HIP_TRY(hipGetLastError());
    clear_error();
    return CL_OK;
}

extern "C" int32_t cl_set_kernel_timing(int32_t enable)
{
    if (enable && !g_timing.a) {
        HIP_TRY(hipEventCreate(&g_timing.a));
        HIP_TRY(hipEventCreate(&g_timing.b));
    }
    g_timing.on = enable != 0;
    g_timing.valid = false;
    return CL_OK;
}

extern "C" int32_t cl_last_kernel_ms(float *ms, int32_t *launches)
{
    if (!ms || !launches) return fail(CL_EINVAL, "null argument");
    if (!g_timing.on || !g_timing.valid) return fail(CL_EINVAL, "no timed forward call yet");
    HIP_TRY(hipEventSynchronize(g_timing.b));
    HIP_TRY(hipEventElapsedTime(ms, g_timing.a, g_timing.b));
    *launches = g_timing.launches;
    return CL_OK;
}

namespace {

// Launch shape of the convolution path: the batch is cut into groups of images whose
// column matrices (one per filter group) stay under kConvXtCap bytes; each group of
// images is one launch of the MFMA path over the block rows of all filter groups.
constexpr size_t kConvXtCap = (size_t)1024 << 20;

struct ConvPlan {
    ConvGeom cg{};
    int OCg = 0, panels_per_group = 0, imgs = 0;
    bool gather = false;       // blocks decoded once per call, no column matrix in memory: conv_mfma_kernel
    int groups_at_once = 1;    // filter groups per launch: all of them, or one (the compact form)
    size_t lds = 0, xt_bytes = 0, part_bytes = 0, wt_bytes = 0, rows_bytes = 0;
    size_t total() const { return xt_bytes + part_bytes + wt_bytes + rows_bytes; }
};

// From this many columns on (image x output pixel) the fp32 path decodes the layer's
// blocks once per call into dense tiles in the workspace, and a multiply kernel of its own
// gathers each 128 x 128 piece of the column matrix into LDS straight from the input, so
// that the column matrix never exists in memory.  Below, and for calls too small to
// give that kernel's one tile width enough work items (see plan_conv), the column matrix
// is written out and the blocks of a column tile are decoded inside the multiply kernel
// (measured on the AlexNet and VGG-16 convolutions at 1 to 64 images: with these limits
// the gathered form is the faster one wherever it is taken, by 4-25 %).
constexpr int64_t kConvGatherColumns = 512;

// compact: the form that needs the least scratch - filter groups one after the other
// through the same buffers, blocks decoded inside the multiply kernel.
int32_t plan_conv(const cl_layer *L, const cl_conv_desc *cv, int batch, bool bf16, const DeviceLimits &dl, ConvPlan &P,
                  bool compact = false)
{
    if (!cv) return fail(CL_EINVAL, "null convolution descriptor");
    if (cv->C < 1 || cv->H < 1 || cv->W < 1 || cv->R < 1 || cv->S < 1 || cv->stride < 1 || cv->pad < 0 || cv->groups < 1 ||
        cv->out_channels < 1)
        return fail(CL_EINVAL, "bad convolution geometry");
    if (cv->C % cv->groups || cv->out_channels % cv->groups) return fail(CL_EINVAL, "groups must divide C and out_channels");
    ConvGeom &g = P.cg;
    g.C = cv->C; g.H = cv->H; g.W = cv->W; g.R = cv->R; g.S = cv->S; g.stride = cv->stride; g.pad = cv->pad;
    g.Cg = cv->C / cv->groups;
    g.P = (cv->H + 2 * cv->pad - cv->R) / cv->stride + 1;
    g.Q = (cv->W + 2 * cv->pad - cv->S) / cv->stride + 1;
    if (g.P < 1 || g.Q < 1) return fail(CL_EINVAL, "filter larger than the padded input");
    if ((int64_t)cv->H * cv->W > INT32_MAX / 2 || (int64_t)g.P * g.Q > kMaxTileColumns || (int64_t)g.Cg * g.R * g.S > INT32_MAX / 2)
        return fail(CL_EUNSUPPORTED, "image planes of more than 2^30 pixels or %d output pixels are not supported", kMaxTileColumns);
    if (L->desc.M != cv->out_channels || L->desc.K != g.Cg * g.R * g.S)
        return fail(CL_EINVAL, "layer is %d x %d, the convolution needs %d x %d", L->desc.M, L->desc.K, cv->out_channels, g.Cg * g.R * g.S);
    if (!mfma_capable(L)) return fail(CL_EUNSUPPORTED, "the convolution path needs blocks of at most %d x %d", kTile, kTile);
    P.OCg = cv->out_channels / cv->groups;
    if (cv->groups > 1 && P.OCg % L->desc.block_h) return fail(CL_EUNSUPPORTED, "block_h %d must divide the %d filters of a group", L->desc.block_h, P.OCg);
    P.panels_per_group = (P.OCg + L->desc.block_h - 1) / L->desc.block_h;
    P.groups_at_once = compact ? 1 : cv->groups;
    const int launch_panels = P.panels_per_group * P.groups_at_once;
    const size_t per_image = (size_t)P.groups_at_once * xt_rows(L) * g.P * g.Q * sizeof(float);
    P.imgs = (int)std::max<size_t>(1, std::min<size_t>((size_t)batch, kConvXtCap / per_image));
    P.lds = mfma_lds_bytes(L, bf16);
    if (P.lds > dl.max_lds) return fail(CL_EUNSUPPORTED, "the convolution path needs %zu bytes of LDS", P.lds);
    const int64_t cols = (int64_t)batch * g.P * g.Q;
    P.gather = !compact && !bf16 && cols >= kConvGatherColumns && (size_t)kConvLdsBytes <= dl.max_lds &&
               // its one tile width must give the chip something to do: work items for a
               // sixteenth of the CUs before the block rows are split, 128 x 128 products for half
               16 * launch_panels * ((cols + kConvColumns - 1) / kConvColumns) >= dl.cus &&
               2 * launch_panels * ((cols + kConvColumns - 1) / kConvColumns) * L->nbw >= dl.cus &&
               (int64_t)(kConvColumns + 1) * g.C * g.H * g.W < (1 << 29) && g.R <= 32 && g.S <= 32;      // the gatherers' 32-bit byte offsets and tap masks
    if (P.gather) {
        // nothing but the launch size limits the images of a launch
        P.imgs = (int)std::min<int64_t>(batch, kMaxTileColumns / ((int64_t)g.P * g.Q));
        P.lds = kConvLdsBytes;
    }
    P.wt_bytes = P.gather ? (size_t)L->n_blocks * kTile * kTile * sizeof(float) : 0;
    P.rows_bytes = P.gather ? round256((size_t)L->nbw * kTile * sizeof(uint2)) : 0;
    // workspace for the larger of a full image group and the last, smaller one
    P.xt_bytes = P.part_bytes = 0;
    for (int imgs : {P.imgs, batch % P.imgs}) {
        if (imgs == 0) continue;
        int nq, np, splits;
        mfma_shape(L, launch_panels, imgs * g.P * g.Q, dl.cus, bf16, nq, np, splits, P.gather, !bf16);
        if (!P.gather) P.xt_bytes = std::max(P.xt_bytes, (size_t)P.groups_at_once * xt_bytes_for(L, np, bf16));
        if (!(P.gather && splits == 1))
            P.part_bytes = std::max(P.part_bytes, (size_t)launch_panels * splits * np * L->desc.block_h * sizeof(float));
    }
    return CL_OK;
}

}  // namespace

extern "C" int32_t cl_conv_workspace_bytes(const cl_layer *L, const cl_conv_desc *cv, int32_t batch, int32_t path, size_t *out)
{
    if (!L || !out) return fail(CL_EINVAL, "null argument");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    if (path != CL_PATH_AUTO && !is_mfma(path)) return fail(CL_EUNSUPPORTED, "convolution runs on the MFMA paths only");
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    ConvPlan P;
    if (int32_t rc = plan_conv(L, cv, batch, path == CL_PATH_MFMA_BF16, dl, P)) return rc;
    *out = P.total();
    return CL_OK;
}

extern "C" int32_t cl_conv_workspace_bytes_min(const cl_layer *L, const cl_conv_desc *cv, int32_t batch, int32_t path, size_t *out)
{
    if (!L || !out) return fail(CL_EINVAL, "null argument");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    if (path != CL_PATH_AUTO && !is_mfma(path)) return fail(CL_EUNSUPPORTED, "convolution runs on the MFMA paths only");
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    ConvPlan P, F;
    if (int32_t rc = plan_conv(L, cv, batch, path == CL_PATH_MFMA_BF16, dl, P, true)) return rc;
    if (int32_t rc = plan_conv(L, cv, batch, path == CL_PATH_MFMA_BF16, dl, F)) return rc;
    *out = std::min(P.total(), F.total());      // the fast form's launch shape can happen to need less
    return CL_OK;
}

namespace {

// One group of images of a convolution call: what the two forms share.
struct ConvCall {
    const cl_layer *L;
    const ConvPlan *P;
    LayerDev D;
    const float *x;         // the group's input, images x C x H x W
    float *y;               // its output, images x M x pq
    const float *bias;
    int ncols, pq, relu;    // columns = images x output pixels
    int launch_panels, nq, Np, splits;
    float *part;
    hipStream_t st;
    bool *timed;            // benchmarks time the first multiply launch of a call
};

// adds the splits of the block rows, bias, activation, NCHW
int32_t conv_finish_splits(const ConvCall &c)
{
    const int ct = reduce_col_tile(c.launch_panels, c.ncols);
    dim3 grid;
    GRID_TRY(grid, (int64_t)c.launch_panels * ((c.ncols + ct - 1) / ct));
    hipLaunchKernelGGL(mfma_reduce_kernel, grid, dim3(256), 0, c.st,
                       c.D, c.part, c.bias, c.y, c.ncols, c.Np, c.splits, c.relu, c.pq, ct, 0, c.L->desc.block_h);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

// The gathered form: one launch gathers the columns and multiplies them with the decoded
// blocks (wt) of all filter groups; it finishes the output itself unless block rows are split.
int32_t conv_gathered(const ConvCall &c, const float *wt, const uint2 *rows, bool combined)
{
    const ConvPlan &P = *c.P;
    const bool direct = c.splits == 1;
    const DirectOut out{direct ? c.y : nullptr, c.bias, c.ncols, c.pq, c.relu};
    // the kernel form for the height of the layer's blocks: how the multiplying wavefronts divide the tile
    const int bh = c.L->desc.block_h, form = bh <= 64 ? 2 : bh <= 96 ? 1 : 0;
    using Kernel = void (*)(LayerDev, const float *, const float *, const uint2 *, float *, ConvGeom, int, int, int, int, DirectOut);
    static const Kernel kernels[6] = {conv_mfma_kernel<false, 1, 4>, conv_mfma_kernel<true, 1, 4>, conv_mfma_kernel<false, 3, 1>,
                                      conv_mfma_kernel<true, 3, 1>,  conv_mfma_kernel<false, 1, 2>, conv_mfma_kernel<true, 1, 2>};
    static LdsLimit seen[6];
    const int which = (combined ? 1 : 0) + 2 * form;
    if (int32_t rc = ensure_lds((const void *)kernels[which], P.lds, seen[which])) return rc;
    dim3 grid;
    GRID_TRY(grid, (int64_t)c.launch_panels * c.splits * (c.Np / kConvColumns));
    if (!*c.timed) timing_begin(c.st);
    hipLaunchKernelGGL(kernels[which], grid, dim3(kConvThreads), P.lds, c.st, c.D, c.x, wt, rows, c.part, P.cg, c.ncols, c.Np, c.splits,
                       P.panels_per_group, out);
    HIP_TRY(hipGetLastError());
    if (!*c.timed) { timing_end(c.st, 1); *c.timed = true; }
    return direct ? CL_OK : conv_finish_splits(c);
}

// The form with the column matrix in memory: P.groups_at_once filter groups per launch of
// each kernel; group grp of a launch has its column matrix at xt + grp * x_bytes and
// multiplies its own block rows.
int32_t conv_columns(ConvCall c, int groups_total, bool bf16, void *xt)
{
    const ConvPlan &P = *c.P;
    const cl_layer *L = c.L;
    const size_t x_bytes = xt_bytes_for(L, c.Np, bf16);
    for (int grp0 = 0; grp0 < groups_total; grp0 += P.groups_at_once) {
        const unsigned groups = (unsigned)P.groups_at_once;
        c.D.panel0 = grp0 * P.panels_per_group;
        if (bf16)
            hipLaunchKernelGGL(im2col_split_kernel, dim3((unsigned)std::min((c.Np + 63) / 64, 4096), (unsigned)(L->nbw * 8), groups), dim3(256), 0,
                               c.st, c.x, (uint16_t *)xt, P.cg, x_bytes / sizeof(uint16_t), c.ncols, c.Np, L->desc.block_w, L->desc.K,
                               xb_plane_elems(L, c.Np), grp0);
        else {
            // rows per workgroup: as many (up to kIm2colRows) as leave a couple of thousand workgroups
            const int64_t col_wgs = std::min((c.Np / 4 + 255) / 256, 4096);
            int rpw = kIm2colRows;
            while (rpw > 1 && col_wgs * (L->nbw * kTile / rpw) * groups < 2048) rpw >>= 1;
            hipLaunchKernelGGL(im2col_pad_kernel, dim3((unsigned)col_wgs, (unsigned)(L->nbw * kTile / rpw), groups), dim3(256), 0, c.st,
                               c.x, (float *)xt, P.cg, x_bytes / sizeof(float), c.ncols, c.Np, L->desc.block_w, L->desc.K, grp0, rpw);
        }
        HIP_TRY(hipGetLastError());
        if (!*c.timed) timing_begin(c.st);
        // block rows that are not split need no adding up: the multiply kernel finishes the output
        const bool direct = !bf16 && c.splits == 1;
        const DirectOut out{direct ? c.y : nullptr, c.bias, c.ncols, c.pq, c.relu};
        if (int32_t rc = launch_mfma(L, c.D, bf16, c.nq, c.launch_panels, c.splits, c.Np, P.panels_per_group, x_bytes, P.lds, xt, c.part, c.st, out))
            return rc;
        if (!*c.timed) { timing_end(c.st, 1); *c.timed = true; }
        if (!direct)
            if (int32_t rc = conv_finish_splits(c)) return rc;
    }
    return CL_OK;
}

}  // namespace

extern "C" int32_t cl_compressed_conv_forward(const cl_layer *L, const cl_conv_desc *cv, const float *d_X,
                                              const float *d_bias, float *d_Y, int32_t batch, int32_t relu,
                                              int32_t path, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (int32_t rc = require_device(L)) return rc;
    if (!d_X || !d_Y) return fail(CL_EINVAL, "null activation pointer");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    if (path != CL_PATH_AUTO && !is_mfma(path)) return fail(CL_EUNSUPPORTED, "convolution runs on the MFMA paths only");
    if ((uintptr_t)d_workspace % 256) return fail(CL_EINVAL, "workspace must be 256-byte aligned");
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    const bool bf16 = path == CL_PATH_MFMA_BF16;
    // the fast form if the workspace holds it, else the compact one
    ConvPlan P;
    if (int32_t rc = plan_conv(L, cv, batch, bf16, dl, P)) return rc;
    if (workspace_bytes < P.total() || !d_workspace) {
        const size_t fast = P.total();
        P = ConvPlan{};
        if (int32_t rc = plan_conv(L, cv, batch, bf16, dl, P, true)) return rc;
        if (workspace_bytes < P.total() || !d_workspace)
            return fail(CL_EINVAL, "workspace too small: %zu < %zu (%zu for the fast form)", workspace_bytes, P.total(), fast);
    }
    hipStream_t st = (hipStream_t)stream;
    const ConvGeom &g = P.cg;
    // the workspace: column matrices (not in the gathered form), partial tiles, decoded blocks, row table
    char *ws = (char *)d_workspace;
    void *xt = ws;
    float *part = (float *)(ws + P.xt_bytes);
    float *wt = (float *)(ws + P.xt_bytes + P.part_bytes);
    uint2 *rows = (uint2 *)(ws + P.xt_bytes + P.part_bytes + P.wt_bytes);
    const bool combined = g.R * g.S <= 32;      // one tap mask per column instead of one per filter row and one per filter column
    if (P.gather) {
        const size_t lds = table_image_bytes(L->val_lut_bits, L->idx_lut_bits, 1 << L->desc.weight_bits) + (size_t)kWTileBytes;
        static LdsLimit seen;
        if (int32_t rc = ensure_lds((const void *)decode_tiles_kernel, lds, seen)) return rc;
        // n_blocks workgroups of kTileDecodeThreads threads: more threads than the row table has entries
        hipLaunchKernelGGL(decode_tiles_kernel, dim3((unsigned)L->n_blocks), dim3(kTileDecodeThreads), lds, st, make_dev(L), wt, g, L->nbw * kTile,
                           combined ? 1 : 0, rows);
        HIP_TRY(hipGetLastError());
    }
    bool timed = false;
    ConvCall c{L, &P, make_dev(L), nullptr, nullptr, d_bias, 0, g.P * g.Q, relu, P.panels_per_group * P.groups_at_once, 0, 0, 0, part, st, &timed};
    for (int b0 = 0; b0 < batch; b0 += P.imgs) {
        const int nb = std::min(P.imgs, batch - b0);
        c.ncols = nb * c.pq;
        mfma_shape(L, c.launch_panels, c.ncols, dl.cus, bf16, c.nq, c.Np, c.splits, P.gather, !bf16);
        c.x = d_X + (size_t)b0 * g.C * g.H * g.W;
        c.y = d_Y + (size_t)b0 * L->desc.M * c.pq;
        if (int32_t rc = P.gather ? conv_gathered(c, wt, rows, combined) : conv_columns(c, cv->groups, bf16, xt)) return rc;
    }
    clear_error();
    return CL_OK;
}
