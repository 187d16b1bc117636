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
    const uint32_t *val_mlut;
    const uint32_t *idx_mlut;
    int M, K, bh, bw, nbw;
    int val_mbits, idx_mbits, ncode;
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
    d.val_mlut = L->dev.val_mlut;
    d.idx_mlut = L->dev.idx_mlut;
    d.M = L->desc.M;
    d.K = L->desc.K;
    d.bh = L->desc.block_h;
    d.bw = L->desc.block_w;
    d.nbw = L->nbw;
    d.val_mbits = L->val_mbits;
    d.idx_mbits = L->idx_mbits;
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

// Fields of a multi-symbol decode-table entry (two layouts, see the host builder).
template <bool WIDE>
struct Entry {
    static constexpr int SB = WIDE ? 8 : 6;      // bits per symbol
    static constexpr int CAP = WIDE ? 2 : 3;     // symbols per entry
    static constexpr int AT = SB * CAP;
    static constexpr uint32_t SM = (1u << SB) - 1u;
    static __device__ __forceinline__ uint32_t sym(uint32_t e, int j) { return (e >> (SB * j)) & SM; }
    static __device__ __forceinline__ uint32_t bits(uint32_t e) { return (e >> AT) & 15u; }
    static __device__ __forceinline__ uint32_t count(uint32_t e) { return (e >> (AT + 4)) & 3u; }
    static __device__ __forceinline__ uint32_t first_bits(uint32_t e) { return (e >> (AT + 6)) & 15u; }
    static __device__ __forceinline__ uint32_t sym_sum(uint32_t e)
    {
        uint32_t t = sym(e, 0) + sym(e, 1);
        if (CAP > 2) t += sym(e, 2);
        return t;
    }
};

// Staging arrays of one wavefront: one slot per entry plus one spare slot per lane
// that swallows the stores of absent symbols.
constexpr int kStage = CL_MAX_CHUNK_ENTRIES + 64;

// What a lane holds of its chunk before decoding starts.
struct ChunkRaw {
    cl_chunk_meta m;
    uint32_t next_off;
    uint32_t w0, w1, w2;
    int gap;
};

// 128-bit read of the lane's 64-bit slice plus the start of the next one, the
// lane's gap nibble and the chunk's table record.
__device__ __forceinline__ ChunkRaw load_chunk(const LayerDev &L, uint32_t c, int lane)
{
    ChunkRaw r;
    r.m = L.meta[c];
    r.next_off = L.meta[c + 1].sym_off;
    uint32_t w[4];
    __builtin_memcpy(w, L.payload + (size_t)c * kChunkBytes + lane * 8, 16);
    r.w0 = w[0];
    r.w1 = w[1];
    r.w2 = w[2];
    const uint32_t gbyte = L.gaps[(size_t)c * kGapBytes + (lane >> 1)];
    r.gap = (int)((gbyte >> (4 * (lane & 1))) & 15u);
    return r;
}

struct ChunkInfo {
    uint32_t e0;      // first entry
    int n;            // entries in the chunk
    uint32_t blk0;    // block of the first entry
    uint32_t pos0;    // position carry of that block
};

// Decode tables in LDS.
struct Tables {
    const uint32_t *vm, *im;
    const float *cb;
};

// Huffman-decode a chunk (Algorithm 2 steps 5-6 for the span of the streams the
// chunk holds) and prefix-sum its relative indices (step 7) in one go.  On return
// the wavefront's LDS staging arrays hold, in entry order,
//   vs[i]  the value index of entry i
//   ss[i]  sum of (z + 1) over entries 0..i of the chunk (inclusive)
// Pass 1 counts codewords and sums z + 1 per lane; one wavefront scan of the
// packed pair gives every lane its first output slot and its starting sum; pass 2
// decodes again straight into place.  Both passes take several symbols per table
// lookup while a whole index still lies inside the lane's slice, then finish one
// symbol at a time.
template <typename E_T, bool WIDE>
__device__ __forceinline__ ChunkInfo decode_chunk(const LayerDev &L, const ChunkRaw &raw, int lane,
                                                  const Tables &T, E_T *vs, E_T *ss)
{
    using En = Entry<WIDE>;
    ChunkInfo ci;
    ci.e0 = raw.m.sym_off;
    ci.n = (int)(raw.next_off - raw.m.sym_off);
    ci.blk0 = raw.m.blk0;
    ci.pos0 = raw.m.pos0;
    const int nv = (raw.m.val_bits + 63) >> 6;
    const bool is_val = lane < nv;
    const int slice = is_val ? lane : lane - nv;
    const int sub_bits = is_val ? (int)raw.m.val_bits : (int)raw.m.idx_bits;
    const int limit = min(64, sub_bits - slice * 64);
    const int mbits = is_val ? L.val_mbits : L.idx_mbits;
    const uint32_t mask = (1u << mbits) - 1u;
    const uint32_t *mlut = is_val ? T.vm : T.im;
    const int mlimit = limit - mbits;      // a whole-index lookup at pos <= mlimit stays inside the slice
    const uint32_t w0 = raw.w0, w1 = raw.w1, w2 = raw.w2;

    // ---- pass 1: how many codewords start in this slice, how far they advance the position
    uint32_t cnt = 0, adv = 0;
    int pos = raw.gap;
    while (pos <= mlimit) {
        const uint32_t e = mlut[window_bits(w0, w1, w2, pos) & mask];
        const uint32_t n = En::count(e);
        pos += (int)En::bits(e);
        cnt += n;
        adv += En::sym_sum(e) + n;
    }
    while (pos < limit) {
        const uint32_t e = mlut[window_bits(w0, w1, w2, pos) & mask];
        pos += (int)En::first_bits(e);
        adv += En::sym(e, 0) + 1u;
        ++cnt;
    }
    // ---- counts (value + index lanes: <= 2048 in total, 12 bits) and advances (<= 2^18) share one scan
    const uint32_t mine = cnt | ((is_val ? 0u : adv) << 12);
    const uint32_t incl = wave_incl_scan(mine);
    const uint32_t total_val = nv > 0 ? ((uint32_t)__builtin_amdgcn_readlane((int)incl, nv - 1) & 0xfffu) : 0u;
    const uint32_t total_all = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63) & 0xfffu;
    if (total_val > (uint32_t)CL_MAX_CHUNK_ENTRIES || total_all - total_val > (uint32_t)CL_MAX_CHUNK_ENTRIES ||
        ci.n > CL_MAX_CHUNK_ENTRIES) {
        ci.n = 0;                           // not a chunk this library wrote: skip it
        return ci;
    }
    const uint32_t excl = incl - mine;
    uint32_t off = (excl & 0xfffu) - (is_val ? 0u : total_val);
    uint32_t run = excl >> 12;
    // ---- pass 2: decode into place.  A value lane stores the symbols themselves, a
    // relative-index lane stores the running sum after each symbol.
    E_T *dst = is_val ? vs : ss;
    const uint32_t keep = is_val ? 0u : 0xffffffffu, inc = is_val ? 0u : 1u;
    const uint32_t spare = (uint32_t)CL_MAX_CHUNK_ENTRIES + (uint32_t)lane;
    pos = raw.gap;
    while (pos <= mlimit) {
        const uint32_t e = mlut[window_bits(w0, w1, w2, pos) & mask];
        const uint32_t n = En::count(e);
        pos += (int)En::bits(e);
        const uint32_t t0 = (run & keep) + En::sym(e, 0) + inc;
        const uint32_t t1 = (t0 & keep) + En::sym(e, 1) + inc;
        dst[off] = (E_T)t0;
        dst[n > 1u ? off + 1u : spare] = (E_T)t1;
        run = n > 1u ? t1 : t0;
        if (En::CAP > 2) {
            const uint32_t t2 = (t1 & keep) + En::sym(e, 2) + inc;
            dst[n > 2u ? off + 2u : spare] = (E_T)t2;
            run = n > 2u ? t2 : run;
        }
        off += n;
    }
    while (pos < limit) {
        const uint32_t e = mlut[window_bits(w0, w1, w2, pos) & mask];
        pos += (int)En::first_bits(e);
        run = (run & keep) + En::sym(e, 0) + inc;
        dst[off] = (E_T)run;
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

__device__ __forceinline__ BlockGeom block_geom(const LayerDev &L, uint32_t b)
{
    BlockGeom g;
    g.b = b;
    const int brow = (int)(b / (uint32_t)L.nbw);
    g.row_id = brow * L.bh;
    g.col_id = (int)(b - (uint32_t)brow * (uint32_t)L.nbw) * L.bw;
    g.bhp = min(L.bh, L.M - g.row_id);
    g.bwp = min(L.bw, L.K - g.col_id);
    g.shift = (g.bhp & (g.bhp - 1)) == 0 ? (31 - __builtin_clz((uint32_t)g.bhp)) : -1;
    return g;
}

// Position inside a block -> (row, column) offsets; column-major inside the block.
__device__ __forceinline__ void split_pos(uint32_t pos, const BlockGeom &g, uint32_t &r, uint32_t &c)
{
    if (g.bwp == 1) { r = pos; c = 0; }
    else if (g.shift >= 0) { c = pos >> g.shift; r = pos & ((uint32_t)g.bhp - 1u); }
    else { c = pos / (uint32_t)g.bhp; r = pos - c * (uint32_t)g.bhp; }
}

// Walk the chunk block by block.  Inside block b the position of entry i is the
// chunk-wide running sum ss[i] plus `base` minus 1: the carry restarts with each
// block, and the first block of a chunk continues from the chunk table's carry.
// seg(g, base, i0, i1) is called once per (block, entry range) by all lanes.
template <typename E_T, class F>
__device__ __forceinline__ void for_each_segment(const LayerDev &L, const ChunkInfo &ci, const E_T *ss, F &&seg)
{
    uint32_t b = ci.blk0;
    int i0 = 0;
    const int n = ci.n;
    while (i0 < n) {
        uint32_t bend = L.block_ptr[b + 1];
        while (bend <= ci.e0 + (uint32_t)i0) bend = L.block_ptr[++b + 1];   // finished or empty blocks
        const int i1 = (int)min((uint32_t)n, bend - ci.e0);
        const uint32_t base = i0 == 0 ? ci.pos0 : 0u - (uint32_t)ss[i0 - 1];
        seg(block_geom(L, b), base, i0, i1);
        i0 = i1;
    }
}

// LDS carve-up shared by the chunk kernels.
template <typename E_T>
struct Smem {
    Tables T;
    E_T *stage;         // per wavefront: vs[kStage] then ss[kStage]
    float *extra;
};

static size_t smem_fixed_bytes(int vmbits, int imbits, int ncode, size_t e_bytes)
{
    return (((size_t)1 << vmbits) + ((size_t)1 << imbits)) * sizeof(uint32_t) + (size_t)ncode * 4 +
           (size_t)kWaves * 2 * kStage * e_bytes;
}

template <typename E_T>
__device__ __forceinline__ Smem<E_T> carve(uint8_t *base, const LayerDev &L)
{
    Smem<E_T> s;
    uint32_t *vm = (uint32_t *)base;
    uint32_t *im = vm + (1 << L.val_mbits);
    float *cb = (float *)(im + (1 << L.idx_mbits));
    s.T.vm = vm;
    s.T.im = im;
    s.T.cb = cb;
    s.stage = (E_T *)(cb + L.ncode);
    s.extra = (float *)(s.stage + kWaves * 2 * kStage);
    return s;
}

// Both tables have at least 2^10 entries, so they are whole numbers of 16-byte rows.
template <typename E_T>
__device__ __forceinline__ void load_tables(const Smem<E_T> &s, const LayerDev &L)
{
    const int nv4 = (1 << L.val_mbits) / 4, ni4 = (1 << L.idx_mbits) / 4;
    const uint4 *gv = (const uint4 *)L.val_mlut, *gi = (const uint4 *)L.idx_mlut;
    uint4 *sv = (uint4 *)s.T.vm, *si = (uint4 *)s.T.im;
    for (int t = threadIdx.x; t < nv4 + ni4; t += blockDim.x) {
        if (t < nv4) sv[t] = gv[t];
        else si[t - nv4] = gi[t - nv4];
    }
    float *cb = (float *)s.T.cb;
    for (int t = threadIdx.x; t < L.ncode; t += blockDim.x) cb[t] = L.codebook[t];
}

// ------------------------------------------------------------------------- //
// decode_layer: symbols and (optionally) the dense matrix
// ------------------------------------------------------------------------- //
template <typename E_T, bool WIDE>
__global__ __launch_bounds__(kThreads) void decode_kernel(LayerDev L, uint8_t *val_out, uint8_t *idx_out, float *dense)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem<E_T> s = carve<E_T>(smem_raw, L);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const uint32_t c = blockIdx.x * kWaves + (uint32_t)wave;
    const bool have = c < L.n_chunks;
    ChunkRaw raw{};
    if (have) raw = load_chunk(L, c, lane);
    load_tables(s, L);
    __syncthreads();
    if (!have) return;
    E_T *vs = s.stage + (size_t)wave * 2 * kStage;
    E_T *ss = vs + kStage;
    const ChunkInfo ci = decode_chunk<E_T, WIDE>(L, raw, lane, s.T, vs, ss);
    for_each_segment<E_T>(L, ci, ss, [&](const BlockGeom &g, uint32_t base, int i0, int i1) {
        for (int i = i0 + lane; i < i1; i += 64) {
            const uint32_t e = ci.e0 + (uint32_t)i;
            const uint32_t v = vs[i];
            const uint32_t sum = ss[i];
            const uint32_t pos = sum + base - 1u;
            if (val_out) val_out[e] = (uint8_t)v;
            if (idx_out) idx_out[e] = (uint8_t)(sum - (i ? (uint32_t)ss[i - 1] : 0u) - 1u);
            if (dense && v != 0 && pos < (uint32_t)g.bhp * (uint32_t)g.bwp) {
                uint32_t r, cc;
                split_pos(pos, g, r, cc);
                dense[(size_t)(g.row_id + (int)r) * L.K + (size_t)(g.col_id + (int)cc)] = s.T.cb[v];
            }
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
// Columns of activations a workgroup may stage in LDS per image.
constexpr int kXCap = 640;
// Largest batch tile that stages its activations in LDS.
constexpr int kXldsMaxBt = 4;

// Workgroup j of block row p takes chunks [8 j, 8 j + 8) of that block row, one per
// wavefront, and accumulates w * x into an LDS tile of the bh x BT outputs of the
// block row (Algorithm 2 step 12, b[row_id : row_id + bh, :] += block * a[col_id :
// col_id + bw, :]), then adds the tile into Y.  Each lane takes one entry per
// round.  With XLDS the activation columns the workgroup's chunks can touch are
// staged in LDS first (when they fit kXCap); otherwise they are read from global
// memory one round ahead.
template <typename E_T, bool WIDE, int BT, bool XLDS>
__global__ __launch_bounds__(kThreads) void fc_sparse_kernel(LayerDev L, const float *__restrict__ X, float *Y,
                                                             int wg_per_panel)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem<E_T> s = carve<E_T>(smem_raw, L);
    const int p = (int)(blockIdx.x / (uint32_t)wg_per_panel), j = (int)(blockIdx.x % (uint32_t)wg_per_panel);
    const uint32_t pc1 = L.panel_chunk[p + 1];
    const uint32_t my0 = L.panel_chunk[p] + (uint32_t)j * kWaves;
    if (my0 >= pc1) return;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const uint32_t c = my0 + (uint32_t)wave;
    const bool have = c < pc1;
    ChunkRaw raw{};
    if (have) raw = load_chunk(L, c, lane);
    const int row_id = p * L.bh;
    const int bhp = min(L.bh, L.M - row_id);
    float *ytile = s.extra;                  // [BT][bh]
    float *xs = ytile + (size_t)L.bh * BT;   // [BT][kXCap] when XLDS
    for (int t = threadIdx.x; t < L.bh * BT; t += blockDim.x) ytile[t] = 0.0f;
    // activation columns this workgroup's chunks can touch: from the first chunk's
    // first block to the block the next workgroup starts in (or the block row's end)
    int col_a = 0;
    bool slab = false;
    if (XLDS) {
        const uint32_t c_end = min(pc1, my0 + (uint32_t)kWaves);
        const uint32_t b_a = L.meta[my0].blk0;
        const uint32_t b_b = c_end < pc1 ? L.meta[c_end].blk0 : (uint32_t)(p + 1) * (uint32_t)L.nbw - 1u;
        col_a = (int)(b_a - (uint32_t)p * (uint32_t)L.nbw) * L.bw;
        const int col_b = min(L.K, (int)(b_b - (uint32_t)p * (uint32_t)L.nbw + 1u) * L.bw);
        const int width = col_b - col_a;
        slab = width <= kXCap;
        if (slab) {
#pragma unroll
            for (int b = 0; b < BT; ++b)
                for (int t = threadIdx.x; t < width; t += blockDim.x) xs[b * kXCap + t] = X[(size_t)b * L.K + col_a + t];
        }
    }
    load_tables(s, L);
    __syncthreads();
    if (have) {
        E_T *vs = s.stage + (size_t)wave * 2 * kStage;
        E_T *ss = vs + kStage;
        const ChunkInfo ci = decode_chunk<E_T, WIDE>(L, raw, lane, s.T, vs, ss);
        struct Round {
            bool act;
            uint32_t r;
            float w;
            float x[BT];
        };
        for_each_segment<E_T>(L, ci, ss, [&](const BlockGeom &g, uint32_t base, int i0, int i1) {
            const uint32_t np = (uint32_t)g.bhp * (uint32_t)g.bwp;
            auto fetch = [&](int at) {
                Round q;
                const int i = at + lane;
                const bool in = i < i1;
                const uint32_t v = in ? vs[i] : 0u;
                const uint32_t pos = (in ? (uint32_t)ss[i] : 1u) + base - 1u;
                q.act = v != 0 && pos < np;
                uint32_t cc = 0;
                q.r = 0;
                if (q.act) split_pos(pos, g, q.r, cc);
                q.w = s.T.cb[v];
                const int col = g.col_id + (int)cc;
                if (XLDS && slab) {
#pragma unroll
                    for (int b = 0; b < BT; ++b) q.x[b] = xs[b * kXCap + (col - col_a)];
                } else {
#pragma unroll
                    for (int b = 0; b < BT; ++b) q.x[b] = q.act ? X[(size_t)b * L.K + col] : 0.0f;
                }
                return q;
            };
            Round cur = fetch(i0);
            for (int at = i0; at < i1; at += 64) {
                Round nxt = cur;
                if (at + 64 < i1) nxt = fetch(at + 64);
                if (cur.act) {
                    float *y = ytile + cur.r;
#pragma unroll
                    for (int b = 0; b < BT; ++b) atomicAdd(y + b * L.bh, cur.w * cur.x[b]);
                }
                cur = nxt;
            }
        });
    }
    __syncthreads();
    for (int t = threadIdx.x; t < bhp * BT; t += blockDim.x) {
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

void release_device(cl_layer *L)
{
    if (L->dev.blob) {
        (void)hipFree(L->dev.blob);
        L->dev = DeviceImage{};
    }
}

// The running position sum inside a chunk is at most entries * 2^k.
static bool sums_fit_u16(const cl_layer *L) { return ((int64_t)CL_MAX_CHUNK_ENTRIES << L->desc.index_bits) <= 65535; }

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
        {L->val_mlut.data(), L->val_mlut.size() * 4, 0},
        {L->idx_mlut.data(), L->idx_mlut.size() * 4, 0},
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
    L->dev.val_mlut = (const uint32_t *)(blob + secs[6].off);
    L->dev.idx_mlut = (const uint32_t *)(blob + secs[7].off);
    clear_error();
    return CL_OK;
}

extern "C" int32_t cl_decode_layer(const cl_layer *L, uint8_t *d_val_sym, uint8_t *d_idx_sym,
                                   uint32_t *d_block_ptr, float *d_dense, void *stream)
{
    if (int32_t rc = require_device(L)) return rc;
    hipStream_t st = (hipStream_t)stream;
    const LayerDev D = make_dev(L);
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    if (d_block_ptr)
        HIP_TRY(hipMemcpyAsync(d_block_ptr, L->dev.block_ptr, (size_t)(L->n_blocks + 1) * 4, hipMemcpyDeviceToDevice, st));
    if (d_dense) {
        const size_t n = (size_t)L->desc.M * L->desc.K;
        hipLaunchKernelGGL(fill_kernel, dim3((unsigned)std::min<size_t>((n + 255) / 256, 4096)), dim3(256), 0, st, d_dense, n, 0.0f);
        HIP_TRY(hipGetLastError());
    }
    if (L->n_chunks > 0 && (d_val_sym || d_idx_sym || d_dense)) {
        const bool narrow = sums_fit_u16(L);
        const size_t lds = smem_fixed_bytes(D.val_mbits, D.idx_mbits, D.ncode, narrow ? 2 : 4);
        const dim3 grid((unsigned)((L->n_chunks + kWaves - 1) / kWaves));
        if (lds > dl.max_lds) return fail(CL_EUNSUPPORTED, "decode tables need %zu bytes of LDS", lds);
#define CL_LAUNCH_DECODE(E, W)                                                                                      \
    do {                                                                                                            \
        if (lds > 64 * 1024)                                                                                        \
            HIP_TRY(hipFuncSetAttribute((const void *)decode_kernel<E, W>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
        hipLaunchKernelGGL((decode_kernel<E, W>), grid, dim3(kThreads), lds, st, D, d_val_sym, d_idx_sym, d_dense); \
    } while (0)
        if (narrow && !L->wide) CL_LAUNCH_DECODE(uint16_t, false);
        else if (narrow) CL_LAUNCH_DECODE(uint16_t, true);
        else if (!L->wide) CL_LAUNCH_DECODE(uint32_t, false);
        else CL_LAUNCH_DECODE(uint32_t, true);
#undef CL_LAUNCH_DECODE
        HIP_TRY(hipGetLastError());
    }
    clear_error();
    return CL_OK;
}


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
        const bool narrow = sums_fit_u16(L);
        const size_t fixed = smem_fixed_bytes(D.val_mbits, D.idx_mbits, D.ncode, narrow ? 2 : 4);
        // LDS per image: a column of the output tile, plus the staged activations for small tiles
        auto lds_for = [&](int bt) { return fixed + (size_t)L->desc.block_h * 4 * bt + (bt <= kXldsMaxBt ? (size_t)kXCap * 4 * bt : 0); };
        // largest power-of-two batch tile (<= 16) that fits; prefer to stay under 64 KiB
        size_t budget = std::min<size_t>(dl.max_lds, 64 * 1024);
        if (lds_for(1) > budget) budget = dl.max_lds;
        if (lds_for(1) > budget) return fail(CL_EUNSUPPORTED, "block_h %d needs more LDS than a workgroup has", L->desc.block_h);
        int bt_max = 16;
        while (bt_max > 1 && lds_for(bt_max) > budget) bt_max >>= 1;
        // one wavefront per chunk: each block row gets enough workgroups for its chunks
        const int wg_per_panel = (int)((L->max_panel_chunks + kWaves - 1) / kWaves);
        const dim3 grid((unsigned)(L->n_panels * wg_per_panel));
        timing_begin(st);
        int launches = 0;
        for (int b0 = 0; b0 < batch; ++launches) {
            int bt = bt_max;
            while (bt > batch - b0) bt >>= 1;
            const size_t lds = lds_for(bt);
            const float *x = d_X + (size_t)b0 * K;
            float *y = d_Y + (size_t)b0 * M;
#define CL_LAUNCH_SPARSE(E, W, BTV)                                                                                \
    do {                                                                                                           \
        auto kern = fc_sparse_kernel<E, W, BTV, (BTV <= kXldsMaxBt)>;                                             \
        if (lds > 64 * 1024)                                                                                       \
            HIP_TRY(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
        hipLaunchKernelGGL(kern, grid, dim3(kThreads), lds, st, D, x, y, wg_per_panel);                           \
    } while (0)
#define CL_LAUNCH_SPARSE_BT(E, W)                                   \
    switch (bt) {                                                   \
    case 16: CL_LAUNCH_SPARSE(E, W, 16); break;                     \
    case 8: CL_LAUNCH_SPARSE(E, W, 8); break;                       \
    case 4: CL_LAUNCH_SPARSE(E, W, 4); break;                       \
    case 2: CL_LAUNCH_SPARSE(E, W, 2); break;                       \
    default: CL_LAUNCH_SPARSE(E, W, 1); break;                      \
    }
            if (narrow && !L->wide) { CL_LAUNCH_SPARSE_BT(uint16_t, false) }
            else if (narrow) { CL_LAUNCH_SPARSE_BT(uint16_t, true) }
            else if (!L->wide) { CL_LAUNCH_SPARSE_BT(uint32_t, false) }
            else { CL_LAUNCH_SPARSE_BT(uint32_t, true) }
#undef CL_LAUNCH_SPARSE_BT
#undef CL_LAUNCH_SPARSE
            HIP_TRY(hipGetLastError());
            b0 += bt;
        }
        timing_end(st, launches);
    }
    if (relu) {
        hipLaunchKernelGGL(relu_kernel, dim3((unsigned)std::min<size_t>((nout + 255) / 256, 2048)), dim3(256), 0, st, d_Y, nout);
        HIP_TRY(hipGetLastError());
    }
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

extern "C" int32_t cl_conv_workspace_bytes(const cl_layer *, const cl_conv_desc *, int32_t, int32_t, size_t *)
{
    return fail(CL_EUNSUPPORTED, "convolution forward is not built yet");
}

extern "C" int32_t cl_compressed_conv_forward(const cl_layer *, const cl_conv_desc *, const float *, const float *,
                                              float *, int32_t, int32_t, int32_t, void *, size_t, void *)
{
    return fail(CL_EUNSUPPORTED, "convolution forward is not built yet");
}
