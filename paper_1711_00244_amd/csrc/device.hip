// gfx950 kernels and their launchers: chunk-parallel Huffman decode, position
// prefix sums, codebook lookup, and the fused sparse-weight x dense-activation
// product (Algorithm 2 of the paper, re-cast for 64-lane wavefronts).
//
// One wavefront owns one 4096-bit chunk.  Lane l owns bits [64 l, 64 l + 64) of
// it; the chunk table tells which lanes hold value-index codewords and which hold
// relative-index codewords, and the lane-gap table tells each lane where its first
// codeword starts.  Decode tables live in LDS.  A first pass counts codewords per
// lane, a wavefront prefix sum turns counts into output slots, a second pass
// decodes into those slots.  Positions come from a second wavefront prefix sum
// over (z + 1), restarted at block boundaries.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>

#include "layer.hpp"

namespace cl {

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(CL_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

constexpr int kWaves = 8;                 // wavefronts per workgroup in the chunk kernels
constexpr int kThreads = kWaves * 64;

// Everything a kernel needs to read a layer, passed by value.
struct LayerDev {
    const uint8_t *payload;
    const cl_chunk_meta *meta;
    const uint8_t *gaps;
    const uint32_t *block_ptr;
    const uint32_t *panel_chunk;
    const float *codebook;
    const lut_t *val_lut;
    const lut_t *idx_lut;
    int M, K, bh, bw, nbw;
    int val_lut_bits, idx_lut_bits, ncode;
    uint32_t n_chunks;
};

static LayerDev make_dev(const cl_layer *L)
{
    LayerDev d;
    d.payload = L->dev.payload;
    d.meta = L->dev.meta;
    d.gaps = L->dev.gaps;
    d.block_ptr = L->dev.block_ptr;
    d.panel_chunk = L->dev.panel_chunk;
    d.codebook = L->dev.codebook;
    d.val_lut = L->dev.val_lut;
    d.idx_lut = L->dev.idx_lut;
    d.M = L->desc.M;
    d.K = L->desc.K;
    d.bh = L->desc.block_h;
    d.bw = L->desc.block_w;
    d.nbw = L->nbw;
    d.val_lut_bits = L->val_lut_bits;
    d.idx_lut_bits = L->idx_lut_bits;
    d.ncode = 1 << L->desc.weight_bits;
    d.n_chunks = (uint32_t)L->n_chunks;
    return d;
}

// ------------------------------------------------------------------------- //
// wavefront primitives
// ------------------------------------------------------------------------- //
// Inclusive add-scan over the 64 lanes (all lanes must be active): four shifts
// inside each row of 16 lanes, then the row totals are carried across rows.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1,3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2,3
    return v;
}

__device__ __forceinline__ uint32_t wave_last(uint32_t v) { return (uint32_t)__builtin_amdgcn_readlane((int)v, 63); }

// Orders this wavefront's LDS writes before its later LDS reads by other lanes.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The next decode-table index at bit `pos` (0..63) of a lane's window.  w0,w1 are
// the lane's own 64 bits, w2 the first 32 bits of the following slice.
__device__ __forceinline__ uint32_t window_bits(uint32_t w0, uint32_t w1, uint32_t w2, int pos)
{
    const uint32_t lo = pos < 32 ? w0 : w1;
    const uint32_t hi = pos < 32 ? w1 : w2;
    return __builtin_amdgcn_alignbit(hi, lo, (uint32_t)pos & 31u);
}

struct ChunkInfo {
    uint32_t e0;      // first entry
    int n;            // entries in the chunk
    uint32_t blk0;    // block of the first entry
    uint32_t pos0;    // position carry of that block
};

// Huffman-decode chunk c into the wavefront's LDS staging arrays vs[] (value
// indices) and zs[] (relative indices), both in entry order.
// Algorithm 2 steps 5-6, for the span of the streams this chunk holds.
__device__ __forceinline__ ChunkInfo decode_chunk(const LayerDev &L, uint32_t c, int lane,
                                                  const lut_t *s_vlut, const lut_t *s_ilut,
                                                  uint8_t *vs, uint8_t *zs)
{
    const cl_chunk_meta m = L.meta[c];
    ChunkInfo ci;
    ci.e0 = m.sym_off;
    ci.n = (int)(L.meta[c + 1].sym_off - m.sym_off);
    ci.blk0 = m.blk0;
    ci.pos0 = m.pos0;
    const int nv = (m.val_bits + 63) >> 6;

    // 128-bit read of the lane's slice and the start of the next one
    uint32_t w[4];
    __builtin_memcpy(w, L.payload + (size_t)c * kChunkBytes + lane * 8, 16);
    const uint32_t gbyte = L.gaps[(size_t)c * kGapBytes + (lane >> 1)];
    const int gap = (int)((gbyte >> (4 * (lane & 1))) & 15u);

    const bool is_val = lane < nv;
    const int slice = is_val ? lane : lane - nv;
    const int sub_bits = is_val ? (int)m.val_bits : (int)m.idx_bits;
    const int limit = min(64, sub_bits - slice * 64);
    const lut_t *lut = is_val ? s_vlut : s_ilut;
    const uint32_t mask = (1u << (is_val ? L.val_lut_bits : L.idx_lut_bits)) - 1u;

    // pass 1: codewords that start in this lane's slice
    uint32_t cnt = 0;
    for (int pos = gap; pos < limit;) {
        const uint32_t e = lut[window_bits(w[0], w[1], w[2], pos) & mask];
        pos += (int)(e >> 8);
        ++cnt;
    }
    // counts -> output slots
    const uint32_t incl = wave_incl_scan(cnt);
    const uint32_t total_val = nv > 0 ? (uint32_t)__builtin_amdgcn_readlane((int)incl, nv - 1) : 0u;
    uint32_t off = incl - cnt - (is_val ? 0u : total_val);
    // pass 2: decode into place
    uint8_t *dst = is_val ? vs : zs;
    for (int pos = gap; pos < limit;) {
        const uint32_t e = lut[window_bits(w[0], w[1], w[2], pos) & mask];
        pos += (int)(e >> 8);
        if (off < (uint32_t)CL_MAX_CHUNK_ENTRIES) dst[off] = (uint8_t)(e & 0xffu);
        ++off;
    }
    wave_lds_fence();
    return ci;
}

struct BlockGeom {
    uint32_t b;
    int row_id, col_id, bhp, bwp;
    int shift;        // log2(bhp) when bhp is a power of two, else -1
};

// Visit every entry of a decoded chunk with its position inside its block
// (Algorithm 1 step 7: prefix sum of the relative indices; each entry advances the
// position by z + 1, the carry restarts with each block).
// f(active, v, pos, geom, entry_index) is called by all 64 lanes together.
template <class F>
__device__ __forceinline__ void for_each_entry(const LayerDev &L, const ChunkInfo &ci, int lane,
                                               const uint8_t *vs, const uint8_t *zs, F &&f)
{
    uint32_t b = ci.blk0;
    uint32_t carry = ci.pos0;
    int i0 = 0;
    const int n = min(ci.n, CL_MAX_CHUNK_ENTRIES);
    while (i0 < n) {
        uint32_t bend = L.block_ptr[b + 1];
        while (bend <= ci.e0 + (uint32_t)i0) {      // block finished (or empty): next block, carry restarts
            ++b;
            carry = 0;
            bend = L.block_ptr[b + 1];
        }
        const int seg_end = (int)min((uint32_t)n, bend - ci.e0);
        BlockGeom g;
        g.b = b;
        const int brow = (int)(b / (uint32_t)L.nbw);
        g.row_id = brow * L.bh;
        g.col_id = (int)(b - (uint32_t)brow * (uint32_t)L.nbw) * L.bw;
        g.bhp = min(L.bh, L.M - g.row_id);
        g.bwp = min(L.bw, L.K - g.col_id);
        g.shift = (g.bhp & (g.bhp - 1)) == 0 ? (31 - __builtin_clz((uint32_t)g.bhp)) : -1;
        for (int base = i0; base < seg_end; base += 64) {
            const int i = base + lane;
            const bool act = i < seg_end;
            const uint32_t v = act ? vs[i] : 0u;
            const uint32_t z1 = act ? (uint32_t)zs[i] + 1u : 0u;
            const uint32_t s = wave_incl_scan(z1);
            const uint32_t pos = carry + s - 1u;
            carry += wave_last(s);
            f(act, v, pos, g, ci.e0 + (uint32_t)i);
        }
        i0 = seg_end;
    }
}

// Position inside a block -> (row, column) offsets; column-major inside the block.
__device__ __forceinline__ void split_pos(uint32_t pos, const BlockGeom &g, uint32_t &r, uint32_t &c)
{
    if (g.bwp == 1) { r = pos; c = 0; }
    else if (g.shift >= 0) { c = pos >> g.shift; r = pos & ((uint32_t)g.bhp - 1u); }
    else { c = pos / (uint32_t)g.bhp; r = pos - c * (uint32_t)g.bhp; }
}

// LDS carve-up shared by the chunk kernels.
struct Smem {
    lut_t *vlut;
    lut_t *ilut;
    float *cb;
    uint8_t *stage;     // kWaves * 2 * CL_MAX_CHUNK_ENTRIES
    float *extra;
};

__host__ __device__ inline size_t smem_fixed_bytes(int vbits, int ibits, int ncode)
{
    return ((size_t)1 << vbits) * sizeof(lut_t) + ((size_t)1 << ibits) * sizeof(lut_t) + (size_t)ncode * 4 +
           (size_t)kWaves * 2 * CL_MAX_CHUNK_ENTRIES;
}

__device__ __forceinline__ Smem carve(uint8_t *base, const LayerDev &L)
{
    Smem s;
    s.vlut = (lut_t *)base;
    s.ilut = s.vlut + (1 << L.val_lut_bits);
    s.cb = (float *)(s.ilut + (1 << L.idx_lut_bits));
    s.stage = (uint8_t *)(s.cb + L.ncode);
    s.extra = (float *)(s.stage + kWaves * 2 * CL_MAX_CHUNK_ENTRIES);
    return s;
}

__device__ __forceinline__ void load_tables(const Smem &s, const LayerDev &L)
{
    // both tables are a whole number of dwords (at least 2 entries each)
    const uint32_t *gv = (const uint32_t *)L.val_lut, *gi = (const uint32_t *)L.idx_lut;
    uint32_t *sv = (uint32_t *)s.vlut, *si = (uint32_t *)s.ilut;
    for (int t = threadIdx.x; t < (1 << L.val_lut_bits) / 2; t += blockDim.x) sv[t] = gv[t];
    for (int t = threadIdx.x; t < (1 << L.idx_lut_bits) / 2; t += blockDim.x) si[t] = gi[t];
    for (int t = threadIdx.x; t < L.ncode; t += blockDim.x) s.cb[t] = L.codebook[t];
}

// ------------------------------------------------------------------------- //
// decode_layer: symbols and (optionally) the dense matrix
// ------------------------------------------------------------------------- //
__global__ __launch_bounds__(kThreads) void decode_kernel(LayerDev L, uint8_t *val_out, uint8_t *idx_out, float *dense)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    load_tables(s, L);
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const uint32_t c = blockIdx.x * kWaves + (uint32_t)wave;
    if (c >= L.n_chunks) return;
    uint8_t *vs = s.stage + (size_t)wave * 2 * CL_MAX_CHUNK_ENTRIES;
    uint8_t *zs = vs + CL_MAX_CHUNK_ENTRIES;
    const ChunkInfo ci = decode_chunk(L, c, lane, s.vlut, s.ilut, vs, zs);
    for_each_entry(L, ci, lane, vs, zs, [&](bool act, uint32_t v, uint32_t pos, const BlockGeom &g, uint32_t e) {
        if (!act) return;
        if (val_out) val_out[e] = (uint8_t)v;
        if (idx_out) idx_out[e] = zs[e - ci.e0];
        if (dense && v != 0 && pos < (uint32_t)g.bhp * (uint32_t)g.bwp) {
            uint32_t r, cc;
            split_pos(pos, g, r, cc);
            dense[(size_t)(g.row_id + (int)r) * L.K + (size_t)(g.col_id + (int)cc)] = s.cb[v];
        }
    });
}

__global__ void fill_kernel(float *p, size_t n, float v)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// ------------------------------------------------------------------------- //
// fused decode + sparse multiply (small batches)
// ------------------------------------------------------------------------- //
// Workgroup (panel p, split j) decodes its share of the chunks of block row p and
// accumulates w * x into an LDS tile of the bh x B outputs of that block row
// (Algorithm 2 step 12, b[row_id : row_id + bh, :] += block * a[col_id : col_id + bw, :]),
// then adds the tile into Y.
__global__ __launch_bounds__(kThreads) void fc_sparse_kernel(LayerDev L, const float *__restrict__ X, float *Y,
                                                             int B, int splits)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    const int p = (int)(blockIdx.x / (uint32_t)splits), j = (int)(blockIdx.x % (uint32_t)splits);
    const uint32_t pc0 = L.panel_chunk[p], pc1 = L.panel_chunk[p + 1];
    const uint32_t nck = pc1 - pc0;
    const uint32_t my0 = pc0 + (uint32_t)(((uint64_t)nck * (uint32_t)j) / (uint32_t)splits);
    const uint32_t my1 = pc0 + (uint32_t)(((uint64_t)nck * (uint32_t)(j + 1)) / (uint32_t)splits);
    if (my0 >= my1) return;
    const int row_id = p * L.bh;
    const int bhp = min(L.bh, L.M - row_id);
    float *ytile = s.extra;      // [B][bh]
    for (int t = threadIdx.x; t < L.bh * B; t += blockDim.x) ytile[t] = 0.0f;
    load_tables(s, L);
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    uint8_t *vs = s.stage + (size_t)wave * 2 * CL_MAX_CHUNK_ENTRIES;
    uint8_t *zs = vs + CL_MAX_CHUNK_ENTRIES;
    for (uint32_t c = my0 + (uint32_t)wave; c < my1; c += kWaves) {
        const ChunkInfo ci = decode_chunk(L, c, lane, s.vlut, s.ilut, vs, zs);
        for_each_entry(L, ci, lane, vs, zs, [&](bool act, uint32_t v, uint32_t pos, const BlockGeom &g, uint32_t) {
            if (!act || v == 0 || pos >= (uint32_t)g.bhp * (uint32_t)g.bwp) return;
            uint32_t r, cc;
            split_pos(pos, g, r, cc);
            const float w = s.cb[v];
            const float *x = X + (size_t)(g.col_id + (int)cc);
            float *y = ytile + r;
            for (int b = 0; b < B; ++b) atomicAdd(y + (size_t)b * L.bh, w * x[(size_t)b * L.K]);
        });
        wave_lds_fence();    // staging is reused by the next chunk
    }
    __syncthreads();
    for (int t = threadIdx.x; t < bhp * B; t += blockDim.x) {
        const int b = t / bhp, r = t - b * bhp;
        const float v = ytile[b * L.bh + r];
        if (v != 0.0f) atomicAdd(Y + (size_t)b * L.M + row_id + r, v);
    }
}

// Y[b][m] = bias[m] (or 0) before the partial sums are added in.
__global__ void init_out_kernel(float *Y, const float *bias, int M, int B)
{
    const size_t n = (size_t)M * B;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        Y[i] = bias ? bias[i % (size_t)M] : 0.0f;
}

__global__ void relu_kernel(float *Y, size_t n)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        Y[i] = fmaxf(Y[i], 0.0f);
}

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
    release_device(L);
    struct Sec { const void *src; size_t bytes; size_t off; };
    Sec secs[8] = {
        {L->payload.data(), L->payload.size(), 0},
        {L->meta.data(), L->meta.size() * sizeof(cl_chunk_meta), 0},
        {L->gaps.data(), L->gaps.size(), 0},
        {L->block_ptr.data(), L->block_ptr.size() * 4, 0},
        {L->panel_chunk.data(), L->panel_chunk.size() * 4, 0},
        {L->codebook.data(), L->codebook.size() * 4, 0},
        {L->val_lut.data(), L->val_lut.size() * sizeof(lut_t), 0},
        {L->idx_lut.data(), L->idx_lut.size() * sizeof(lut_t), 0},
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
    L->dev.payload = (const uint8_t *)(blob + secs[0].off);
    L->dev.meta = (const cl_chunk_meta *)(blob + secs[1].off);
    L->dev.gaps = (const uint8_t *)(blob + secs[2].off);
    L->dev.block_ptr = (const uint32_t *)(blob + secs[3].off);
    L->dev.panel_chunk = (const uint32_t *)(blob + secs[4].off);
    L->dev.codebook = (const float *)(blob + secs[5].off);
    L->dev.val_lut = (const lut_t *)(blob + secs[6].off);
    L->dev.idx_lut = (const lut_t *)(blob + secs[7].off);
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
        const size_t lds = smem_fixed_bytes(D.val_lut_bits, D.idx_lut_bits, D.ncode);
        const unsigned grid = (unsigned)((L->n_chunks + kWaves - 1) / kWaves);
        hipLaunchKernelGGL(decode_kernel, dim3(grid), dim3(kThreads), lds, st, D, d_val_sym, d_idx_sym, d_dense);
        HIP_TRY(hipGetLastError());
    }
    clear_error();
    return CL_OK;
}

namespace {
// Largest batch tile whose output tile fits beside the tables in LDS.
int sparse_batch_tile(const cl_layer *L, size_t lds_budget, int batch)
{
    const size_t fixed = smem_fixed_bytes(L->val_lut_bits, L->idx_lut_bits, 1 << L->desc.weight_bits);
    if (fixed + (size_t)L->desc.block_h * 4 > lds_budget) return 0;
    const size_t per_image = (size_t)L->desc.block_h * 4;
    return (int)std::min<size_t>((size_t)batch, (lds_budget - fixed) / per_image);
}
}  // namespace

extern "C" int32_t cl_fc_workspace_bytes(const cl_layer *L, int32_t batch, int32_t path, size_t *out)
{
    if (!L || !out) return fail(CL_EINVAL, "null argument");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    if (path != CL_PATH_AUTO && path != CL_PATH_SPARSE && path != CL_PATH_MFMA_F32) return fail(CL_EINVAL, "unknown path %d", path);
    *out = 0;
    return CL_OK;
}

extern "C" int32_t cl_compressed_fc_forward(const cl_layer *L, const float *d_X, const float *d_bias,
                                            float *d_Y, int32_t batch, int32_t relu, int32_t path,
                                            void *d_workspace, size_t workspace_bytes, void *stream)
{
    (void)d_workspace;
    if (int32_t rc = require_device(L)) return rc;
    if (!d_X || !d_Y) return fail(CL_EINVAL, "null activation pointer");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    size_t need = 0;
    if (int32_t rc = cl_fc_workspace_bytes(L, batch, path, &need)) return rc;
    if (workspace_bytes < need) return fail(CL_EINVAL, "workspace too small: %zu < %zu", workspace_bytes, need);
    if (path == CL_PATH_MFMA_F32) return fail(CL_EUNSUPPORTED, "MFMA path is not built yet");
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    hipStream_t st = (hipStream_t)stream;
    const LayerDev D = make_dev(L);
    const int M = L->desc.M, K = L->desc.K;
    const size_t nout = (size_t)M * batch;

    hipLaunchKernelGGL(init_out_kernel, dim3((unsigned)std::min<size_t>((nout + 255) / 256, 2048)), dim3(256), 0, st,
                       d_Y, d_bias, M, batch);
    HIP_TRY(hipGetLastError());
    if (L->n_chunks > 0) {
        const size_t budget = std::min<size_t>(dl.max_lds, 64 * 1024);
        int bt = sparse_batch_tile(L, budget, batch);
        if (bt < 1) bt = sparse_batch_tile(L, dl.max_lds, batch);
        if (bt < 1) return fail(CL_EUNSUPPORTED, "block_h %d needs more LDS than a workgroup has", L->desc.block_h);
        const size_t fixed = smem_fixed_bytes(D.val_lut_bits, D.idx_lut_bits, D.ncode);
        // enough workgroups to fill the chip twice over, at least one per block row
        const int target = std::max(1, dl.cus) * 2;
        const int64_t mean_chunks = std::max<int64_t>(1, L->n_chunks / std::max(1, L->n_panels));
        int splits = (int)std::max<int64_t>(1, std::min<int64_t>((target + L->n_panels - 1) / L->n_panels, mean_chunks));
        for (int b0 = 0; b0 < batch; b0 += bt) {
            const int nb = std::min(bt, batch - b0);
            const size_t lds = fixed + (size_t)L->desc.block_h * nb * 4;
            if (lds > 64 * 1024)
                HIP_TRY(hipFuncSetAttribute((const void *)fc_sparse_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(fc_sparse_kernel, dim3((unsigned)(L->n_panels * splits)), dim3(kThreads), lds, st,
                               D, d_X + (size_t)b0 * K, d_Y + (size_t)b0 * M, nb, splits);
            HIP_TRY(hipGetLastError());
        }
    }
    if (relu) {
        hipLaunchKernelGGL(relu_kernel, dim3((unsigned)std::min<size_t>((nout + 255) / 256, 2048)), dim3(256), 0, st, d_Y, nout);
        HIP_TRY(hipGetLastError());
    }
    clear_error();
    return CL_OK;
}

extern "C" int32_t cl_conv_workspace_bytes(const cl_layer *, const cl_conv_desc *, int32_t, int32_t, size_t *)
{
    return fail(CL_EUNSUPPORTED, "convolution forward is not built yet");
}

extern "C" int32_t cl_compressed_conv_forward(const cl_layer *, const cl_conv_desc *, const float *, const float *,
                                              float *, int32_t, int32_t, int32_t, void *, size_t, void *)
{
    return fail(CL_EUNSUPPORTED, "convolution forward is not built yet");
}
