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
#include <hip/hip_runtime.h>
#include <type_traits>

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstring>

#include "layer.hpp"

namespace cl {

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess) return fail(CL_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
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
    const float *codebook;
    const lut_t *val_lut;
    const lut_t *idx_lut;
    int M, K, bh, bw, nbw;
    int val_bits, idx_bits, ncode;       // index widths of the decode tables, codebook entries
    int table_rows;                      // 16-byte rows of the table image (tables + codebook)
    uint32_t n_chunks;
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

// Largest value over the 64 lanes (all lanes must be active), the same in every lane
// and known to be uniform.
__device__ __forceinline__ uint32_t wave_max(uint32_t v)
{
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// W consecutive floats (W * 4-byte aligned) with one load.
template <int W> __device__ __forceinline__ void load_floats(const float *p, float *dst)
{
    typedef float vec_t __attribute__((ext_vector_type(W)));
    const vec_t v = *(const vec_t *)p;
#pragma unroll
    for (int i = 0; i < W; ++i) dst[i] = v[i];
}

template <> __device__ __forceinline__ void load_floats<1>(const float *p, float *dst) { dst[0] = *p; }

// Decode tables and codebook in LDS.
struct Tables {
    const lut_t *vlut;
    const lut_t *ilut;
    const float *cb;
    uint32_t vmask, imask;
};

// A lane's record, split into its two spans.
struct LaneRecord {
    uint64_t vbuf;     // value-index codewords, next codeword at bit 0
    uint64_t ibuf;     // relative-index codewords, next codeword at bit 0
    uint32_t n;        // entries in the record (0 for lanes beyond the chunk)
};

struct ChunkHead {
    cl_chunk_meta m;
    uint32_t nrec;
};

__device__ __forceinline__ ChunkHead load_head(const LayerDev &L, uint32_t c)
{
    ChunkHead h;
    h.m = L.meta[c];
    h.nrec = L.meta[c + 1].rec_off - h.m.rec_off;
    return h;
}

__device__ __forceinline__ LaneRecord load_record(const LayerDev &L, const ChunkHead &h, int lane)
{
    LaneRecord r;
    const uint64_t w = (uint32_t)lane < h.nrec ? L.records[(size_t)h.m.rec_off + lane] : 0ull;
    r.n = (uint32_t)w & 15u;
    r.vbuf = w >> kCountBits;
    r.ibuf = __builtin_bitreverse64(w);
    return r;
}

// One table lookup: the entry for the codeword at the head of buf (symbol in its second
// byte); buf moves on to the next codeword.  The entry itself is the shift amount
// (length in its low bits, the shifter ignores the rest), which keeps the loop-carried
// chain at mask, address, read, shift.
__device__ __forceinline__ uint32_t next_entry(uint64_t &buf, const lut_t *lut, uint32_t mask)
{
    const uint32_t e = lut[(uint32_t)buf & mask];
    buf >>= (e & 63u);
    return e;
}

constexpr int kMaxEntries = 15;        // a record's count field is four bits

// A lane's record with both codeword streams decoded: eight bits per entry, entry j in
// byte j % 4 of word j / 4; the bytes of entries the record does not have are zero.
struct Symbols {
    uint32_t z[4];     // relative indices
    uint32_t v[4];     // value indices
    uint32_t n;        // entries
    uint32_t nmax;     // largest n of the wavefront (uniform)
    uint32_t adv;      // sum of (z + 1): how far the record moves the position
};

// One step of the decoding pass: entry J of both streams.  Every lane looks up (the
// masked table index is always inside the table) and stores the symbol, also a lane
// that has no entry J: what it stored is cleared after the pass, so the pass has no
// divergent branch and no per-lane test.
template <int J>
__device__ __forceinline__ void decode_from(LaneRecord &rec, const Tables &T, Symbols &y)
{
    if constexpr (J < kMaxEntries) {
        if ((uint32_t)J >= y.nmax) return;                                  // uniform
        constexpr int at = J % 4;
        // identity selector with 5 at byte `at`: the symbol byte of the table entry goes there
        constexpr uint32_t put = (0x03020100u & ~(0xffu << (8 * at))) | (5u << (8 * at));
        const uint32_t ez = next_entry(rec.ibuf, T.ilut, T.imask);
        const uint32_t ev = next_entry(rec.vbuf, T.vlut, T.vmask);
        y.z[J / 4] = __builtin_amdgcn_perm(ez, y.z[J / 4], put);
        y.v[J / 4] = __builtin_amdgcn_perm(ev, y.v[J / 4], put);
        decode_from<J + 1>(rec, T, y);
    }
}

// Algorithm 2 step 6 for one record: both streams are decoded in one pass - two
// independent table chains per lane, so one lookup's latency hides behind the
// other's - and kept in registers; positions and weights follow from them without
// touching the tables again.  The pass is written out for the fifteen possible entries
// (it ends after the wavefront's longest record), so every byte position is a constant.
// All lanes of the wavefront must be active.
__device__ __forceinline__ Symbols decode_record(LaneRecord rec, const Tables &T)
{
    Symbols y{{0, 0, 0, 0}, {0, 0, 0, 0}, rec.n, wave_max(rec.n), 0};
    decode_from<0>(rec, T, y);
    // clear the bytes of entries a lane does not have: word w keeps its first
    // clamp(n - 4 w, 0, 4) bytes (the shift by 8 bits per byte is done in two halves,
    // so that four bytes shift everything out)
    const uint32_t n4 = 4u * y.n;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if ((uint32_t)(4 * w) >= y.nmax) break;                             // uniform
        const uint32_t half = (uint32_t)min(max((int)n4 - 16 * w, 0), 16);
        const uint32_t drop = (0xffffffffu << half) << half;
        y.z[w] &= ~drop;
        y.v[w] &= ~drop;
    }
    // absent entries are zero bytes: the byte sums of the four words are the sum of z
    uint32_t adv = y.n;
#pragma unroll
    for (int w = 0; w < 4; ++w) adv = __builtin_amdgcn_sad_u8(y.z[w], 0u, adv);
    y.adv = adv;
    return y;
}

struct LaneStart {
    uint32_t entry;    // index, inside the chunk, of the lane's first entry
    uint32_t sum;      // sum of (z + 1) over the block's entries before the lane's first entry
};

// Algorithm 2 step 7: the prefix sum across the wavefront.  Lane counts (<= 15, 960
// per chunk: 10 bits) and lane advances (<= 15 * 256) travel in one scan.
__device__ __forceinline__ LaneStart lane_starts(const Symbols &y, uint32_t pos0)
{
    const uint32_t mine = y.n | (y.adv << 10);
    const uint32_t excl = wave_incl_scan(mine) - mine;
    LaneStart s;
    s.entry = excl & 1023u;
    s.sum = pos0 + (excl >> 10);
    return s;
}

// Calls f(j, v, z, position) for the record's entries in order; sum starts as the
// lane's LaneStart::sum.  Written out like the decoding pass.  With ALL the call is
// made in every lane up to the wavefront's longest record: a lane past its own last
// entry sees v = 0, z = 0 and a position that moves on by one per call (for callers
// to whom a zero weight at such a position does no harm); without, only for the
// lane's own entries.
template <bool ALL, int J, class F>
__device__ __forceinline__ void entries_from(const Symbols &y, uint32_t pos, F &f)
{
    if constexpr (J < kMaxEntries) {
        if ((uint32_t)J >= y.nmax) return;                                  // uniform
        const uint32_t z = (y.z[J / 4] >> (8 * (J % 4))) & 0xffu, v = (y.v[J / 4] >> (8 * (J % 4))) & 0xffu;
        pos += z + 1u;
        if (ALL || (uint32_t)J < y.n) f((uint32_t)J, v, z, pos);
        entries_from<ALL, J + 1>(y, pos, f);
    }
}

template <bool ALL = false, class F>
__device__ __forceinline__ void for_each_entry(const Symbols &y, uint32_t sum, F f)
{
    entries_from<ALL, 0>(y, sum - 1u, f);
}

struct BlockGeom {
    int row_id, col_id, bhp, bwp;
    int shift;        // log2(bwp) when bwp is a power of two, else -1
};

__device__ __forceinline__ BlockGeom block_geom(const LayerDev &L, uint32_t b)
{
    BlockGeom g;
    const int brow = (int)(b / (uint32_t)L.nbw);
    g.row_id = brow * L.bh;
    g.col_id = (int)(b - (uint32_t)brow * (uint32_t)L.nbw) * L.bw;
    g.bhp = min(L.bh, L.M - g.row_id);
    g.bwp = min(L.bw, L.K - g.col_id);
    g.shift = (g.bwp & (g.bwp - 1)) == 0 ? (31 - __builtin_clz((uint32_t)g.bwp)) : -1;
    return g;
}

// Position inside a block -> (row, column) offsets; a block is flattened row by
// row (Algorithm 2 step 9, "arrange as bh x bw block").  The row is clamped so that
// a position beyond the block cannot index outside it.
__device__ __forceinline__ void split_pos(uint32_t pos, const BlockGeom &g, uint32_t &r, uint32_t &c)
{
    if (g.shift >= 0) { r = pos >> g.shift; c = pos & ((uint32_t)g.bwp - 1u); }
    else { r = pos / (uint32_t)g.bwp; c = pos - r * (uint32_t)g.bwp; }
    r = min(r, (uint32_t)g.bhp - 1u);
}

// LDS carve-up shared by the chunk kernels: value table, index table, codebook,
// then kernel-specific space.
struct Smem {
    Tables T;
    float *extra;
};

static size_t smem_fixed_bytes(int vbits, int ibits, int ncode) { return table_image_bytes(vbits, ibits, ncode); }

__device__ __forceinline__ Smem carve(uint8_t *base, const LayerDev &L)
{
    Smem s;
    lut_t *v = (lut_t *)base;
    lut_t *i = v + (1 << L.val_bits);
    // both tables have at least two entries, so they end 4-byte aligned; round up to 16
    const size_t tb = (((size_t)1 << L.val_bits) + ((size_t)1 << L.idx_bits)) * sizeof(lut_t);
    float *cb = (float *)(base + ((tb + 15) & ~(size_t)15));
    s.T.vlut = v;
    s.T.ilut = i;
    s.T.cb = cb;
    s.T.vmask = (1u << L.val_bits) - 1u;
    s.T.imask = (1u << L.idx_bits) - 1u;
    s.extra = cb + ((L.ncode + 3) & ~3);
    return s;
}

// The decode tables and the codebook sit in device memory exactly as they sit in
// LDS (value table, index table, padding to 16 bytes, codebook, padding to 16
// bytes), so a workgroup copies them as 16-byte rows: all loads are issued first,
// the LDS stores follow once the rest of the prologue is under way.
constexpr int kTableRows = 3;            // 16-byte rows per thread: 3 * 512 * 16 B covers two 12-bit tables + codebook

struct TableRegs {
    uint4 row[kTableRows];
};

__device__ __forceinline__ TableRegs fetch_tables(const LayerDev &L)
{
    TableRegs t;
    const uint4 *g = (const uint4 *)L.val_lut;
#pragma unroll
    for (int k = 0; k < kTableRows; ++k) {
        const int i = (int)threadIdx.x + k * kThreads;
        t.row[k] = i < L.table_rows ? g[i] : uint4{0, 0, 0, 0};
    }
    return t;
}

__device__ __forceinline__ void store_tables(const Smem &s, const LayerDev &L, const TableRegs &t)
{
    uint4 *d = (uint4 *)s.T.vlut;
#pragma unroll
    for (int k = 0; k < kTableRows; ++k) {
        const int i = (int)threadIdx.x + k * kThreads;
        if (i < L.table_rows) d[i] = t.row[k];
    }
}

// ------------------------------------------------------------------------- //
// decode_layer: symbols and (optionally) the dense matrix
// ------------------------------------------------------------------------- //
__global__ __launch_bounds__(kThreads) void decode_kernel(LayerDev L, uint8_t *val_out, uint8_t *idx_out, float *dense)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const uint32_t c = blockIdx.x * kWaves + (uint32_t)wave;
    const bool have = c < L.n_chunks;
    ChunkHead h{};
    LaneRecord rec{};
    if (have) {
        h = load_head(L, c);
        rec = load_record(L, h, lane);
    }
    store_tables(s, L, fetch_tables(L));
    __syncthreads();
    if (!have) return;
    const Symbols y = decode_record(rec, s.T);
    const LaneStart st = lane_starts(y, h.m.pos0);
    const BlockGeom g = block_geom(L, h.m.blk);
    const uint32_t e0 = h.m.sym_off + st.entry;
    for_each_entry(y, st.sum, [&](uint32_t j, uint32_t v, uint32_t z, uint32_t pos) {
        if (val_out) val_out[e0 + j] = (uint8_t)v;
        if (idx_out) idx_out[e0 + j] = (uint8_t)z;
        if (dense && v != 0 && pos < (uint32_t)g.bhp * (uint32_t)g.bwp) {
            uint32_t r, cc;
            split_pos(pos, g, r, cc);
            dense[(size_t)(g.row_id + (int)r) * L.K + (size_t)(g.col_id + (int)cc)] = s.T.cb[v];
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
// Workgroup j of block row p takes chunks [8 j, 8 j + 8) of that block row, one per
// wavefront, and accumulates w * x into an LDS tile of the bh x BT outputs of the
// block row (Algorithm 2 step 12, b[row_id : row_id + bh, :] += block * a[col_id :
// col_id + bw, :]); the tile then goes to the workgroup's slot of `part`, and a
// second kernel adds the slots of a block row up.  A lane's entries run along a
// row of the block, so it sums w * x in registers and touches the tile only when
// the row changes.  The activation columns of the blocks the workgroup's chunks
// belong to are staged in LDS first when they fit xcap columns; otherwise they are
// read from global memory.  A padding entry carries codebook value 0 and adds 0.
template <int BT>
__global__ __launch_bounds__(kThreads) void fc_sparse_kernel(LayerDev L, const float *__restrict__ X, float *part,
                                                             int wg_per_panel, int xcap)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    const int p = (int)(blockIdx.x / (uint32_t)wg_per_panel), j = (int)(blockIdx.x % (uint32_t)wg_per_panel);
    const uint32_t pc1 = L.panel_chunk[p + 1];
    const uint32_t my0 = L.panel_chunk[p] + (uint32_t)j * (kWaves * kSparseChunksPerWave);
    if (my0 >= pc1) return;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    // wavefront w takes chunks my0 + w, my0 + 8 + w, ...: all their records are requested
    // before the tables are copied
    bool have[kSparseChunksPerWave];
    ChunkHead h[kSparseChunksPerWave];
    LaneRecord rec[kSparseChunksPerWave];
#pragma unroll
    for (int i = 0; i < kSparseChunksPerWave; ++i) {
        const uint32_t c = my0 + (uint32_t)(i * kWaves + wave);
        have[i] = c < pc1;
        h[i] = ChunkHead{};
        rec[i] = LaneRecord{};
        if (have[i]) {
            h[i] = load_head(L, c);
            rec[i] = load_record(L, h[i], lane);
        }
    }
    const TableRegs tr = fetch_tables(L);
    float *ytile = s.extra;                  // [BT][bh]
    float *xs = ytile + (size_t)L.bh * BT;   // [xcap][BT]: a column's BT images side by side, one LDS read per entry
    // activation columns of the blocks this workgroup's chunks belong to
    const uint32_t pb0 = (uint32_t)p * (uint32_t)L.nbw;
    const uint32_t c_last = min(pc1, my0 + (uint32_t)(kWaves * kSparseChunksPerWave)) - 1u;
    const int col_a = (int)(L.meta[my0].blk - pb0) * L.bw;
    const int col_b = min(L.K, (int)(L.meta[c_last].blk - pb0 + 1u) * L.bw);
    const int width = col_b - col_a;
    const bool slab = width <= xcap;
    if (slab) {
#pragma unroll
        for (int b = 0; b < BT; ++b)
            for (int t = threadIdx.x; t < width; t += blockDim.x) xs[t * BT + b] = X[(size_t)b * L.K + col_a + t];
    }
    for (int t = threadIdx.x; t < L.bh * BT; t += blockDim.x) ytile[t] = 0.0f;
    store_tables(s, L, tr);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kSparseChunksPerWave; ++i) {
        if (!have[i]) continue;
        const Symbols y = decode_record(rec[i], s.T);
        const LaneStart st = lane_starts(y, h[i].m.pos0);
        const BlockGeom g = block_geom(L, h[i].m.blk);
        // The entries of the record in order, in every lane up to the wavefront's longest
        // record: a lane past its own entries multiplies codebook entry 0 with a column
        // of the block.  The instantiations differ in where the activations come from
        // (LDS stays LDS: no generic pointers) and in how a position splits into row and
        // column (shift and mask for a power-of-two block width).
        auto entries = [&](auto load_x, auto split) {
            uint32_t cur = 0;
            float acc[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) acc[b] = 0.0f;
            for_each_entry<true>(y, st.sum, [&](uint32_t, uint32_t v, uint32_t, uint32_t pos) {
                uint32_t r, cc;
                split(pos, r, cc);
                if (r != cur) {
#pragma unroll
                    for (int b = 0; b < BT; ++b) {
                        atomicAdd(ytile + b * L.bh + cur, acc[b]);
                        acc[b] = 0.0f;
                    }
                    cur = r;
                }
                const float w = s.T.cb[v];
                float x[BT];
                load_x((int)cc, x);
#pragma unroll
                for (int b = 0; b < BT; ++b) acc[b] += w * x[b];
            });
#pragma unroll
            for (int b = 0; b < BT; ++b) atomicAdd(ytile + b * L.bh + cur, acc[b]);
        };
        auto with_split = [&](auto load_x) {
            if (g.shift >= 0) {
                const uint32_t sh = (uint32_t)g.shift, cmask = (uint32_t)g.bwp - 1u, rmax = (uint32_t)g.bhp - 1u;
                entries(load_x, [&](uint32_t pos, uint32_t &r, uint32_t &cc) { r = min(pos >> sh, rmax); cc = pos & cmask; });
            } else {
                entries(load_x, [&](uint32_t pos, uint32_t &r, uint32_t &cc) { split_pos(pos, g, r, cc); });
            }
        };
        if (slab) {
            const int xoff = g.col_id - col_a;
            with_split([&](int cc, float (&x)[BT]) {
                constexpr int kW = BT < 4 ? BT : 4;
#pragma unroll
                for (int q = 0; q < BT / kW; ++q) load_floats<kW>(xs + (xoff + cc) * BT + q * kW, x + q * kW);
            });
        } else {
            const float *xg = X + g.col_id;
            with_split([&](int cc, float (&x)[BT]) {
#pragma unroll
                for (int b = 0; b < BT; ++b) x[b] = xg[(size_t)b * L.K + cc];
            });
        }
    }
    __syncthreads();
    float *mine = part + (size_t)blockIdx.x * L.bh * BT;
    for (int t = threadIdx.x; t < L.bh * BT; t += blockDim.x) mine[t] = ytile[t];
}

// Finishes the sparse path: adds up the partial tiles of each block row in a fixed
// order, then bias and activation (Eq. 1): Y[b][row] = act(sum_j part[p][j][b][r] + v[row]).
// One workgroup per (block row, image).  The kernel is a chain of memory latencies and
// nothing else, so it is laid out to have few links: the threads form as many groups
// (slices) as fit next to one pass over the rows, slice s adds slots s, s + slices, ...
// with twelve loads in flight, LDS adds the slices in order.
constexpr int kRedThreads = 512;

__global__ __launch_bounds__(kRedThreads) void fc_reduce_kernel(LayerDev L, const float *__restrict__ part,
                                                                const float *__restrict__ bias, float *Y, int B,
                                                                int part_b, int wg_per_panel, int relu)
{
    __shared__ float slice_sum[kRedThreads];
    const int p = (int)blockIdx.x / B, b = (int)blockIdx.x - p * B;
    const int row_id = p * L.bh;
    const int bhp = min(L.bh, L.M - row_id);
    // the sparse kernel fills one slot per workgroup's worth of chunks of the block row
    constexpr uint32_t kPerWg = kWaves * kSparseChunksPerWave;
    const int active = (int)((L.panel_chunk[p + 1] - L.panel_chunk[p] + kPerWg - 1) / kPerWg);
    const int rows = min(kRedThreads, (bhp + 63) / 64 * 64);        // rows per pass: whole wavefronts
    const int slices = kRedThreads / rows;
    const int sl = (int)threadIdx.x / rows, rl = (int)threadIdx.x - sl * rows;
    // part[p][j][image (part_b of them)][bh]
    const float *src = part + ((size_t)p * wg_per_panel * part_b + b) * L.bh;
    const size_t step = (size_t)part_b * L.bh;
    for (int r0 = 0; r0 < bhp; r0 += rows) {
        const int r = r0 + rl;
        float acc = 0.0f;
        if (r < bhp && sl < slices) {
            // twelve slots per round, all loads issued before the first add (a slot past
            // the last one reads slot sl again and is not added)
            for (int j = sl; j < active; j += 12 * slices) {
                float a[12];
#pragma unroll
                for (int u = 0; u < 12; ++u) {
                    const int jj = j + u * slices;
                    a[u] = src[(size_t)(jj < active ? jj : sl) * step + r];
                }
#pragma unroll
                for (int u = 0; u < 12; ++u)
                    if (j + u * slices < active) acc += a[u];
            }
        }
        if (slices > 1) {
            slice_sum[threadIdx.x] = acc;
            __syncthreads();
            if (sl == 0 && r < bhp)
                for (int k = 1; k < slices; ++k) acc += slice_sum[k * rows + rl];
            __syncthreads();
        }
        if (sl == 0 && r < bhp) {
            if (bias) acc += bias[row_id + r];
            Y[(size_t)b * L.M + row_id + r] = relu ? fmaxf(acc, 0.0f) : acc;
        }
    }
}

// ------------------------------------------------------------------------- //
// large batches: decode a block into a dense LDS tile, multiply on the fp32 MFMA
// ------------------------------------------------------------------------- //
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kTile = 128;               // block rows, block columns and images per workgroup tile

// The activations as the dense-tile kernel reads them: XT[row][b] with the image axis
// padded to Bp (whole image tiles of the kernel) and the K axis laid out block by block, every block
// column of the layer taking kTile rows: row = (k / bw) * kTile + k % bw holds X[b][k],
// the other rows and the padded images are zero.  A wavefront's walk over the blocks
// of a block row is then a walk over consecutive rows whatever the block width.
// kXtTailRows more rows follow (never written; read ahead by the last steps of the last
// block and never multiplied).
constexpr int kBPrefetch = 8;            // k-steps of activations in flight (a multiple of 4 that divides kTile / 2)
constexpr int kXtTailRows = kTile;       // the read-ahead stays within half a block + kBPrefetch rows

__device__ __forceinline__ int xt_row_to_k(int row, int bw, int K)
{
    const int kk = row % kTile, k = (row / kTile) * bw + kk;
    return (kk < bw && k < K) ? k : -1;
}

__global__ __launch_bounds__(256) void transpose_pad_kernel(const float *__restrict__ X, float *XT, int B, int K, int Bp,
                                                            int bw, int rows)
{
    __shared__ float t[32][33];
    const int r0 = blockIdx.x * 32, b0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
    for (int i = ty; i < 32; i += 8) {
        const int b = b0 + i, k = xt_row_to_k(r0 + tx, bw, K);
        t[i][tx] = (b < B && k >= 0) ? X[(size_t)b * K + k] : 0.0f;
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int r = r0 + i, b = b0 + tx;
        if (r < rows && b < Bp) XT[(size_t)r * Bp + b] = t[tx][i];
    }
}

// Sec. III-A: the receptive field of every output pixel becomes a column, so that a
// convolution is the matrix product filters x columns.  Written transposed and
// padded like XT above, row k = (c*R + r)*S + s, column n = image * P*Q + output pixel,
// for the input channels of one group; zero outside the image and past n_cols.
struct ConvGeom {
    int C, H, W, R, S, stride, pad, Cg, P, Q;
};

__global__ __launch_bounds__(256) void im2col_pad_kernel(const float *__restrict__ X, float *XT, ConvGeom cg, size_t x_stride,
                                                         int n_cols, int Np, int bw, int K)
{
    const int c0 = (int)blockIdx.z * cg.Cg;                 // filter group blockIdx.z: its input channels, its matrix
    XT += (size_t)blockIdx.z * x_stride;
    const int k = xt_row_to_k((int)blockIdx.y, bw, K);      // (c, r, s) of this row, or a padding row
    const int s = k % cg.S, r = (k / cg.S) % cg.R, c = k / (cg.S * cg.R);
    const int pq = cg.P * cg.Q;
    const size_t plane = (size_t)cg.H * cg.W;
    const float *xc = X + (size_t)(c0 + c) * plane;         // the row's channel in image 0
    float4 *row = (float4 *)(XT + (size_t)blockIdx.y * Np);
    // a thread writes four consecutive columns (Np is a multiple of the 32-column
    // accumulator): output pixel and image are divided out once and stepped from there
    for (int n4 = blockIdx.x * blockDim.x + threadIdx.x; n4 < Np / 4; n4 += gridDim.x * blockDim.x) {
        float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        const int n = 4 * n4;
        if (k >= 0 && n < n_cols) {
            int img = n / pq;
            const int o = n - img * pq;
            int oy = o / cg.Q, ox = o - oy * cg.Q;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int y = oy * cg.stride - cg.pad + r, x = ox * cg.stride - cg.pad + s;
                if (n + i < n_cols && y >= 0 && y < cg.H && x >= 0 && x < cg.W)
                    v[i] = xc[(size_t)img * cg.C * plane + (size_t)y * cg.W + x];
                if (++ox == cg.Q) {
                    ox = 0;
                    if (++oy == cg.P) { oy = 0; ++img; }
                }
            }
        }
        row[n4] = make_float4(v[0], v[1], v[2], v[3]);
    }
}

// Workgroup (block row p, split j of its blocks, image tile nb) of wavefronts in two roles.
//   Decoders (wavefronts 4 and up, one or two next to each multiplier on a SIMD) decode
//   block i + 1 - a chunk per wavefront, decode / scan / use as in the sparse kernel -
//   and write each entry's weight at its place in a 128 x 128 tile in LDS, row by row
//   (Algorithm 2 steps 5-9: decode, prefix sum, codebook look-up, "arrange as bh x bw
//   block").
//   Multipliers (wavefronts 0-3) multiply block i on the matrix cores (step 12); how
//   the tile and the images are divided among them is the kernel's own business.
// Two weight tiles alternate; a used tile is cleared by the multipliers, so a tile
// is always clean when the decoders get it back.
constexpr int kWStride = kTile + 4;      // floats per weight row of a tile (16-byte rows, 4-bank skew)
constexpr int kWTileBytes = kTile * kWStride * 4;
// The decoder wavefronts' side of the dense-tile kernels: decode the blocks blk_lo ..
// blk_hi - 1 of block row pb0 / nbw into the two alternating 128 x kWStride tiles of
// 32-bit words, one block ahead of the multipliers, meeting them at one barrier per
// block.  The two buffers are BUF_FLOATS floats apart; store(buffer, row, column, v)
// places value index v (the codebook entry, or its two bf16 halves in two half
// tiles).  With CLEAR_BARRIER the multipliers clear a used tile between two barriers
// (their rows are shared), else right after their last read of their own rows.
// Called by wavefronts 4 .. 4 + DEC - 1.
template <int DEC, bool CLEAR_BARRIER, int BUF_FLOATS, class Store>
__device__ __forceinline__ void decoder_role(const LayerDev &L, const Smem &s, float *tiles, int blk_lo, int blk_hi, uint32_t pb0,
                                             int wave, int lane, Store store)
{
    // The chunks of this split's blocks are consecutive, [c_lo, c_hi); decoder
    // d = wave - 4 takes c_lo + d, c_lo + d + DEC, ... and finds a block's
    // end at the first chunk head that names a later block.  Block -> chunk head ->
    // record is a chain of dependent loads, so the stream runs ahead of the decoding:
    // the heads of the next three chunks and the records of the next two are in
    // registers or in flight.  Every load is unconditional (a position past the end
    // re-reads the last chunk and is marked invalid; chunk heads sit in a zero-padded
    // section, so the head after the last one is readable even for a layer without
    // chunks) and nothing touches a loaded value before it is decoded: the loads are
    // not waited for where they are issued.  Heads are read through an address the
    // compiler cannot prove uniform, or they would be moved to scalar registers right
    // behind the load.
    struct Head {
        uint32_t rec_off, rec_end, blk, pos0;
        bool valid;
    };
    uint32_t lane_zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(lane_zero));
    const uint32_t c_hi = blk_lo < blk_hi ? L.block_chunk[pb0 + (uint32_t)blk_hi] : 0u;
    uint32_t c_tail = blk_lo < blk_hi ? L.block_chunk[pb0 + (uint32_t)blk_lo] + (uint32_t)(wave - 4) : 0u;   // next head to load
    auto next_head = [&]() {
        Head h;
        h.valid = c_tail < c_hi;
        const cl_chunk_meta *mp = L.meta + (h.valid ? c_tail : (c_hi ? c_hi - 1u : 0u)) + lane_zero;
        h.rec_off = mp[0].rec_off;
        h.rec_end = mp[1].rec_off;
        h.blk = mp[0].blk;
        h.pos0 = mp[0].pos0;
        c_tail += (uint32_t)DEC;
        return h;
    };
    auto word_of = [&](const Head &h) {
        const uint32_t last = h.rec_end - h.rec_off - 1u;       // a chunk has at least one record
        return L.records[h.rec_off + min((uint32_t)lane, last)];
    };
    Head h0 = next_head(), h1 = next_head(), h2 = next_head();
    uint64_t w0 = word_of(h0), w1 = word_of(h1);
    // decode block bi into a weight tile (clean on entry): Algorithm 2 steps 5-9
    auto produce = [&](int bi, float *tile) {
        const uint32_t b = pb0 + (uint32_t)bi;
        const BlockGeom g = block_geom(L, b);
        while (h0.valid && (uint32_t)__builtin_amdgcn_readfirstlane((int)h0.blk) == b) {
            LaneRecord rec;
            rec.n = (uint32_t)lane < h0.rec_end - h0.rec_off ? (uint32_t)w0 & 15u : 0u;
            rec.vbuf = w0 >> kCountBits;
            rec.ibuf = __builtin_bitreverse64(w0);
            const uint32_t pos0 = h0.pos0;
            // move the stream on; the record load issued here uses a head that arrived
            // a chunk ago
            h0 = h1; w0 = w1;
            h1 = h2; w1 = word_of(h1);
            h2 = next_head();
            const Symbols y = decode_record(rec, s.T);
            const LaneStart st = lane_starts(y, pos0);
            if (g.shift >= 0) {
                // a power-of-two block width (every full block): row and column are a
                // shift and a mask, the column cannot leave the tile, and a padding
                // entry may store its zero (codebook entry 0) like any other
                const uint32_t sh = (uint32_t)g.shift, cmask = (uint32_t)g.bwp - 1u, rmax = (uint32_t)g.bhp - 1u;
                for_each_entry(y, st.sum, [&](uint32_t, uint32_t v, uint32_t, uint32_t pos) {
                    store(tile, min(pos >> sh, rmax), pos & cmask, v);
                });
            } else {
                for_each_entry(y, st.sum, [&](uint32_t, uint32_t v, uint32_t, uint32_t pos) {
                    uint32_t r, cc;
                    split_pos(pos, g, r, cc);
                    if (v != 0 && cc < (uint32_t)kTile) store(tile, r, cc, v);
                });
            }
        }
    };
    // the decoders go first at the issue arbiter: a multiplying wavefront needs one
    // issue slot per 64-cycle multiply, the decoders next to it on the SIMD can have
    // the rest
    __builtin_amdgcn_s_setprio(3);
    __syncthreads();                                    // tables stored, tiles clean
    if (blk_lo < blk_hi) produce(blk_lo, tiles);
    __syncthreads();
    for (int bi = blk_lo; bi < blk_hi; ++bi) {
        if (bi + 1 < blk_hi) produce(bi + 1, tiles + (((bi - blk_lo) & 1) ^ 1) * BUF_FLOATS);
        __syncthreads();
        if (CLEAR_BARRIER) __syncthreads();
    }
}

// NQ = 32 x 32 accumulators per multiplying wavefront = 32-column groups of the
// workgroup's image tile (1, 2, 4 or 8: 32 to 256 images).  A wider tile feeds more
// multiplies from each decoded block; a narrower one wastes fewer padded columns on a
// small batch.  Up to four accumulators a lane's activation values of a k-step are one
// load of NQ floats (accumulator q holds images NQ m + q); with eight they are two
// 16-byte loads, 128 images apart, which leaves registers for four decoder wavefronts
// and four steps of load-ahead.
template <int NQ> struct MfmaShape {
    static constexpr int kDecoders = NQ <= 4 ? 8 : 4;
    static constexpr int kThreads = (4 + kDecoders) * 64;
    static constexpr int kAhead = NQ <= 4 ? kBPrefetch : kBPrefetch / 2;     // k-steps of activations in flight
    static constexpr int kImages = 32 * NQ;
    static constexpr int kVecW = NQ < 4 ? NQ : 4;                             // floats per load
    static constexpr int kVecs = NQ / kVecW;                                  // loads per k-step
};

template <int NQ>
__global__ __launch_bounds__(MfmaShape<NQ>::kThreads) void fc_mfma_kernel(LayerDev L, const float *__restrict__ XT, float *part,
                                                                         int splits, int Bp, int panels_per_x, size_t x_stride)
{
    constexpr int kMfmaDecoders = MfmaShape<NQ>::kDecoders;
    constexpr int kMfmaThreads = MfmaShape<NQ>::kThreads;
    constexpr int kAhead = MfmaShape<NQ>::kAhead;
    constexpr int kImages = MfmaShape<NQ>::kImages;
    constexpr int kVecW = MfmaShape<NQ>::kVecW, kVecs = MfmaShape<NQ>::kVecs;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    float *tiles = (float *)s.extra;                        // [2][kTile rows][kWStride]
    const int nbt = Bp / kImages;
    const int nb = (int)blockIdx.x % nbt;
    const int pj = (int)blockIdx.x / nbt;
    const int p = pj / splits, j = pj % splits;
    // every panels_per_x block rows have an activation matrix of their own, x_stride
    // elements after the one before (the filter groups of a convolution)
    XT += (size_t)(p / panels_per_x) * x_stride;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const bool producer = wave >= 4;
    if (threadIdx.x < kThreads) store_tables(s, L, fetch_tables(L));
    for (int t = threadIdx.x; t < 2 * kWTileBytes / 16; t += kMfmaThreads) ((uint4 *)tiles)[t] = uint4{0, 0, 0, 0};
    // this split's share of the block row's blocks
    const int blk_lo = (int)(((int64_t)L.nbw * j) / splits), blk_hi = (int)(((int64_t)L.nbw * (j + 1)) / splits);
    const uint32_t pb0 = (uint32_t)p * (uint32_t)L.nbw;

    if (producer) {
        decoder_role<kMfmaDecoders, false, kWTileBytes / 4>(L, s, tiles, blk_lo, blk_hi, pb0, wave, lane,
                                                             [&](float *tile, uint32_t r, uint32_t cc, uint32_t v) { tile[__umul24(r, (uint32_t)kWStride) + cc] = s.T.cb[v]; });
        return;
    }

    // Consumer: the A values run as one stream of k-steps over all blocks of this split.
    // With XT laid out block by block, step s of block bi is rows kTile bi + s and
    // kTile bi + 64 + s; the stream is loaded kBPrefetch steps ahead of the multiplies,
    // across block boundaries.  The last steps read ahead into the next rows of XT (the
    // next split's, or the tail rows): valid memory, never multiplied.  The barriers
    // below pair with the decoders' above, one for one.
    floatx16 acc[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) acc[q] = floatx16{0};
    const int kl = lane >> 5, m = lane & 31;
    const float *ap = XT + ((size_t)blk_lo * kTile + 64 * kl) * Bp + (size_t)nb * kImages + kVecW * m;
    const size_t row_stride = (size_t)Bp;
    float aq[kAhead][NQ];
#pragma unroll
    for (int i = 0; i < kAhead; ++i) {
#pragma unroll
        for (int v = 0; v < kVecs; ++v) load_floats<kVecW>(ap + v * kTile, &aq[i][4 * v]);
        ap += row_stride;
    }
    __syncthreads();                                        // tables stored, tiles clean
    __syncthreads();                                        // first block decoded
    for (int bi = blk_lo; bi < blk_hi; ++bi) {
        float *cur = tiles + ((bi - blk_lo) & 1) * (kWTileBytes / 4);
        // B values of four steps: columns 64 kl + 4 g .. + 3 of weight row 32 wave + m
        const float4 *wp = (const float4 *)(cur + (wave * 32 + m) * kWStride + 64 * kl);
        float4 b_cur = wp[0];
        for (int ks = 0; ks < kTile / 2; ks += kAhead) {
            // steps are kept in program order (scheduling barriers): hoisting a group's
            // LDS reads or sinking its loads would put their latency in front of the
            // multiplies
#pragma unroll
            for (int h4 = 0; h4 < kAhead / 4; ++h4) {
                const float4 b_next = wp[min(ks / 4 + h4 + 1, kTile / 8 - 1)];
                __builtin_amdgcn_sched_barrier(0);          // the LDS read goes out before these multiplies
                const float bv[4] = {b_cur.x, b_cur.y, b_cur.z, b_cur.w};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = 4 * h4 + u;
#pragma unroll
                    for (int q = 0; q < NQ; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(aq[i][q], bv[u], acc[q], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);      // the step's A values are free again
#pragma unroll
                    for (int v = 0; v < kVecs; ++v) load_floats<kVecW>(ap + v * kTile, &aq[i][4 * v]);
                    ap += row_stride;
                    __builtin_amdgcn_sched_barrier(0);
                }
                b_cur = b_next;
            }
            // the loads of the group after next start the next block: skip this block's other half
            if (ks == kTile / 2 - 2 * kAhead) ap += (kTile / 2) * row_stride;
        }
        // done with this tile: clear this wavefront's 32 rows of it
        uint4 *z = (uint4 *)(cur + wave * 32 * kWStride);
        for (int t = lane; t < 32 * kWStride / 4; t += 64) z[t] = uint4{0, 0, 0, 0};
        __syncthreads();
    }
    // accumulator 4 v + q, element e of lane l: image 128 v + kVecW (8 (e / 4) + 4 (l / 32) + e % 4) + q
    // of the tile, weight row 32 wave + l % 32; 32 lanes write 32 consecutive floats
    const int r = wave * 32 + m;
    if (r < L.bh) {
        float *mine = part + ((size_t)pj * Bp + (size_t)nb * kImages) * L.bh + r;
#pragma unroll
        for (int v = 0; v < kVecs; ++v) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int slot = 8 * (e / 4) + 4 * kl + (e & 3);
#pragma unroll
                for (int q = 0; q < kVecW; ++q) mine[(size_t)(kTile * v + kVecW * slot + q) * L.bh] = acc[4 * v + q][e];
            }
        }
    }
}

// ------------------------------------------------------------------------- //
// dense tiles on the bf16 matrix cores, three products per fp32 product
// ------------------------------------------------------------------------- //
// A weight w and an activation x are each split into two bf16 terms, w = wh + wl,
// x = xh + xl (round to nearest even; the residual of each is below 2^-18 of the value),
// and w x is taken as xh wh + xh wl + xl wh with fp32 accumulation in
// v_mfma_f32_32x32x16_bf16: three multiplies at sixteen times the fp32 rate.  What is
// dropped (xl wl and the two residuals) is below 3 * 2^-18 of |w x|.
__device__ __forceinline__ uint32_t bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// hi half in the upper 16 bits, lo half in the lower
__device__ __forceinline__ uint32_t bf16_split(float f)
{
    const uint32_t hi = bf16_bits(f);
    const uint32_t lo = bf16_bits(f - __uint_as_float(hi << 16));
    return (hi << 16) | lo;
}

// The activations as the bf16 kernel reads them: two planes (hi, lo) of
// XB[g][column][16] bf16, g = 8 * (block column) + (k % bw) / 16 counting groups of
// sixteen k of the block-ordered K axis (zero beyond a narrow or ragged block and
// beyond the batch), so that the 32 columns of an accumulator are one contiguous
// kilobyte per group.  Each plane has kXbTailGroups more groups (read ahead, never
// multiplied).
constexpr int kXbTailGroups = 4;

__device__ __forceinline__ void store_split4(uint16_t *XB, size_t plane_elems, size_t at, const float v[4])
{
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = bf16_split(v[j]);
    *(uint2 *)(XB + at) = uint2{(w[0] >> 16) | (w[1] & 0xffff0000u), (w[2] >> 16) | (w[3] & 0xffff0000u)};
    *(uint2 *)(XB + plane_elems + at) = uint2{(w[0] & 0xffffu) | (w[1] << 16), (w[2] & 0xffffu) | (w[3] << 16)};
}

// grid: (groups, ceil(Bp / 64)); thread t: column 64 blockIdx.y + t / 4, k quad t % 4
__global__ __launch_bounds__(256) void split_pad_kernel(const float *__restrict__ X, uint16_t *XB, int B, int K, int Bp, int bw,
                                                        size_t plane_elems)
{
    const int g = blockIdx.x, col = blockIdx.y * 64 + (int)(threadIdx.x >> 2), kq = (int)(threadIdx.x & 3);
    if (col >= Bp) return;
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int k = xt_row_to_k((g >> 3) * kTile + (g & 7) * 16 + 4 * kq + j, bw, K);
        v[j] = (k >= 0 && col < B) ? X[(size_t)col * K + k] : 0.0f;
    }
    store_split4(XB, plane_elems, ((size_t)g * Bp + col) * 16 + 4 * kq, v);
}

// the same for a convolution: column = image * P*Q + output pixel, k = (c*R + r)*S + s
__global__ __launch_bounds__(256) void im2col_split_kernel(const float *__restrict__ X, uint16_t *XB, ConvGeom cg, size_t x_stride,
                                                           int n_cols, int Np, int bw, int K, size_t plane_elems)
{
    const int c0 = (int)blockIdx.z * cg.Cg;
    XB += (size_t)blockIdx.z * x_stride;
    const int g = blockIdx.y, kq = (int)(threadIdx.x & 3);
    const int pq = cg.P * cg.Q;
    for (int col = blockIdx.x * 64 + (int)(threadIdx.x >> 2); col < Np; col += gridDim.x * 64) {
        float v[4];
        const int img = col / pq, o = col - img * pq;
        const int y0 = (o / cg.Q) * cg.stride - cg.pad, x0 = (o % cg.Q) * cg.stride - cg.pad;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = xt_row_to_k((g >> 3) * kTile + (g & 7) * 16 + 4 * kq + j, bw, K);
            v[j] = 0.0f;
            if (k >= 0 && col < n_cols) {
                const int s = k % cg.S, r = (k / cg.S) % cg.R, c = k / (cg.S * cg.R);
                const int y = y0 + r, x = x0 + s;
                if (y >= 0 && y < cg.H && x >= 0 && x < cg.W) v[j] = X[(((size_t)img * cg.C + (c0 + c)) * cg.H + y) * cg.W + x];
            }
        }
        store_split4(XB, plane_elems, ((size_t)g * Np + col) * 16 + 4 * kq, v);
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Image tile of 32 NQ columns (NQ = 1, 2, 4, 8).  Unlike the fp32 kernel, whose four
// multiplying wavefronts each take 32 weight rows and all columns, here a wavefront takes
// 32 (64 for NQ = 8) columns and as many of the 128 weight rows as it takes to share the
// tile among four wavefronts: the multiplies are sixteen times faster, and columns read
// once per workgroup instead of four times keep the activation loads off the critical
// path (weights come from LDS).
template <int NQ> struct Bf16Shape {
    static constexpr int kDecoders = 4;
    static constexpr int kThreads = (4 + kDecoders) * 64;
    static constexpr int kAhead = 4;                           // groups of sixteen k in flight
    static constexpr int kImages = 32 * NQ;
    static constexpr int kIT = NQ == 8 ? 2 : 1;                // 32-column groups per wavefront
    static constexpr int kWavesPerCols = NQ >= 4 ? 1 : 4 / NQ; // wavefronts sharing the same columns
    static constexpr int kRT = 4 / kWavesPerCols;              // 32-row tiles per wavefront
};

// Same workgroup roles, barriers, split of the block row and partial-tile layout as
// fc_mfma_kernel.  The decoders store the two bf16 halves of each weight in two half
// tiles; a multiplying wavefront reads the eight hi halves and the eight lo halves of a
// row for a group of sixteen k with one 16-byte LDS read each (lanes 0-31 the first
// eight k, lanes 32-63 the other eight) and feeds three multiplies per accumulator.
constexpr int kHStride = kTile + 8;                       // bf16 per row of a half tile (16-byte rows, 4-bank skew)
constexpr int kBf16BufFloats = 2 * kTile * kHStride / 2;  // floats per buffer: hi tile + lo tile
template <int NQ>
__global__ __launch_bounds__(Bf16Shape<NQ>::kThreads) void fc_mfma_bf16_kernel(LayerDev L, const uint16_t *__restrict__ XB,
                                                                             float *part, int splits, int Bp, size_t plane_elems,
                                                                             int panels_per_x, size_t x_stride)
{
    using S = Bf16Shape<NQ>;
    constexpr int kDec = S::kDecoders, kNThreads = S::kThreads, kAhead = S::kAhead, kImages = S::kImages;
    constexpr int kIT = S::kIT, kRT = S::kRT;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    // two buffers, each a tile of the hi halves and a tile of the lo halves:
    // [2][2][kTile rows][kHStride] bf16
    float *tiles = (float *)s.extra;
    uint32_t *cbp = (uint32_t *)(tiles + 2 * kBf16BufFloats);       // split codebook
    const int nbt = Bp / kImages;
    const int nb = (int)blockIdx.x % nbt;
    const int pj = (int)blockIdx.x / nbt;
    const int p = pj / splits, j = pj % splits;
    XB += (size_t)(p / panels_per_x) * x_stride;            // one pair of planes per filter group
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    store_tables(s, L, fetch_tables(L));
    for (int t = threadIdx.x; t < 2 * kBf16BufFloats / 4; t += kNThreads) ((uint4 *)tiles)[t] = uint4{0, 0, 0, 0};
    for (int t = threadIdx.x; t < L.ncode; t += kNThreads) cbp[t] = bf16_split(L.codebook[t]);
    const int blk_lo = (int)(((int64_t)L.nbw * j) / splits), blk_hi = (int)(((int64_t)L.nbw * (j + 1)) / splits);
    const uint32_t pb0 = (uint32_t)p * (uint32_t)L.nbw;
    if (wave >= 4) {
        decoder_role<kDec, true, kBf16BufFloats>(L, s, tiles, blk_lo, blk_hi, pb0, wave, lane,
                                                 [&](float *tile, uint32_t r, uint32_t cc, uint32_t v) {
                                                     const uint32_t w = cbp[v];
                                                     uint16_t *t16 = (uint16_t *)tile + __umul24(r, (uint32_t)kHStride) + cc;
                                                     t16[0] = (uint16_t)(w >> 16);
                                                     t16[kTile * kHStride] = (uint16_t)w;
                                                 });
        return;
    }

    floatx16 acc[kIT][kRT];
#pragma unroll
    for (int it = 0; it < kIT; ++it)
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) acc[it][rt] = floatx16{0};
    const int kl = lane >> 5, m = lane & 31;
    const int col0 = (wave / S::kWavesPerCols) * kIT * 32;  // this wavefront's first column of the tile
    const int row0 = (wave % S::kWavesPerCols) * kRT * 32;  // and its first weight row
    // group g, column c: 32 bytes at (g Bp + c) * 32, this lane's eight k at + 16 kl
    const uint4 *ap = (const uint4 *)XB + ((size_t)blk_lo * 8 * Bp + (size_t)nb * kImages + col0 + m) * 2 + kl;
    const size_t group_stride = (size_t)Bp * 2, plane_stride = plane_elems / 8;      // in 16-byte units
    uint4 ah[kAhead][kIT], al[kAhead][kIT];
    auto load_group = [&](int slot) {
#pragma unroll
        for (int it = 0; it < kIT; ++it) {
            ah[slot][it] = ap[it * 64];
            al[slot][it] = ap[plane_stride + it * 64];
        }
        ap += group_stride;
    };
#pragma unroll
    for (int i = 0; i < kAhead; ++i) load_group(i);
    __syncthreads();                                        // tables stored, tiles clean
    __syncthreads();                                        // first block decoded
    for (int bi = blk_lo; bi < blk_hi; ++bi) {
        float *buf = tiles + ((bi - blk_lo) & 1) * kBf16BufFloats;
        // the eight hi (lo) halves of row row0 + 32 rt + m for group g: one 16-byte read each
        const uint4 *wp = (const uint4 *)((const uint16_t *)buf + (row0 + m) * kHStride + 8 * kl);
        auto halves_at = [&](int idx, uint4 &h, uint4 &l) {             // idx = g * kRT + rt
            const int g = idx / kRT, rt = idx % kRT;
            h = wp[rt * (32 * kHStride / 8) + 2 * g];
            l = wp[kTile * kHStride / 8 + rt * (32 * kHStride / 8) + 2 * g];
        };
        uint4 bh, bl;
        halves_at(0, bh, bl);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            constexpr int kSlotMask = kAhead - 1;
            const int slot = g & kSlotMask;
#pragma unroll
            for (int rt = 0; rt < kRT; ++rt) {
                const bf16x8 vbh = __builtin_bit_cast(bf16x8, bh), vbl = __builtin_bit_cast(bf16x8, bl);
                if (g * kRT + rt + 1 < 8 * kRT) halves_at(g * kRT + rt + 1, bh, bl);
#pragma unroll
                for (int it = 0; it < kIT; ++it) {
                    const bf16x8 vah = __builtin_bit_cast(bf16x8, ah[slot][it]), val = __builtin_bit_cast(bf16x8, al[slot][it]);
                    acc[it][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vah, vbh, acc[it][rt], 0, 0, 0);
                    acc[it][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vah, vbl, acc[it][rt], 0, 0, 0);
                    acc[it][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(val, vbh, acc[it][rt], 0, 0, 0);
                }
            }
            load_group(slot);
        }
        // every multiplier reads rows that others read too: all done, then each clears a quarter
        __syncthreads();
        uint4 *z = (uint4 *)buf + wave * (kBf16BufFloats / 16);
        for (int t = lane; t < kBf16BufFloats / 16; t += 64) z[t] = uint4{0, 0, 0, 0};
        __syncthreads();
    }
    // accumulator (it, rt), element e of lane l: column col0 + 32 it + 8 (e / 4) + 4 (l / 32) + e % 4
    // of the tile, weight row row0 + 32 rt + l % 32; 32 lanes write 32 consecutive floats
    float *mine = part + ((size_t)pj * Bp + (size_t)nb * kImages + col0) * L.bh;
#pragma unroll
    for (int rt = 0; rt < kRT; ++rt) {
        const int r = row0 + 32 * rt + m;
        if (r >= L.bh) continue;
#pragma unroll
        for (int it = 0; it < kIT; ++it) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int slot = 8 * (e / 4) + 4 * kl + (e & 3);
                mine[(size_t)(32 * it + slot) * L.bh + r] = acc[it][rt][e];
            }
        }
    }
}

// Finishes the dense-tile path: Y = act(sum over the splits of a block row, in a fixed
// order, + bias) (Eq. 1).  A workgroup takes a block row and ct <= kColTile consecutive
// columns (images, or image x output pixel for a convolution): for each split that
// is one contiguous run of ct x bh floats of the partial buffer.  The host picks ct
// so that the launch still has a few workgroups per CU.  FC output
// rows are contiguous in Y[image][row]; a convolution's output is contiguous along
// the pixels, Y[image][row][pixel], so its tile is turned in LDS first.
constexpr int kColTile = 32;

__global__ __launch_bounds__(256) void mfma_reduce_kernel(LayerDev L, const float *__restrict__ part,
                                                          const float *__restrict__ bias, float *Y, int ncols, int part_b,
                                                          int splits, int relu, int conv_pq, int ct)
{
    __shared__ float tile[kColTile][kTile + 1];
    const int ntile = (ncols + ct - 1) / ct;
    const int p = (int)blockIdx.x / ntile, c0 = ((int)blockIdx.x - p * ntile) * ct;
    const int row_id = p * L.bh;
    const int bhp = min(L.bh, L.M - row_id);
    const size_t split_stride = (size_t)part_b * L.bh;
    for (int e = threadIdx.x; e < ct * L.bh; e += blockDim.x) {
        const int ci = e / L.bh, r = e - ci * L.bh;
        const int c = c0 + ci;
        if (c >= ncols || r >= bhp) continue;
        const float *src = part + ((size_t)p * splits * part_b + c) * L.bh + r;
        float t = 0.0f;
        for (int j = 0; j < splits; j += 8) {               // eight loads in flight, added in order
            float a[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) a[u] = src[(size_t)(j + u < splits ? j + u : 0) * split_stride];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (j + u < splits) t += a[u];
        }
        if (bias) t += bias[row_id + r];
        t = relu ? fmaxf(t, 0.0f) : t;
        if (conv_pq == 0) Y[(size_t)c * L.M + row_id + r] = t;
        else tile[ci][r] = t;
    }
    if (conv_pq == 0) return;
    __syncthreads();
    for (int e = threadIdx.x; e < ct * bhp; e += blockDim.x) {
        const int r = e / ct, ci = e - r * ct;
        const int c = c0 + ci;
        if (c < ncols) Y[((size_t)(c / conv_pq) * L.M + row_id + r) * conv_pq + (c % conv_pq)] = tile[ci][r];
    }
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
    // decode tables + codebook, laid out as in LDS
    const int ncode = 1 << L->desc.weight_bits;
    std::vector<char> image(table_image_bytes(L->val_lut_bits, L->idx_lut_bits, ncode), 0);
    {
        const size_t vb = L->val_lut.size() * sizeof(lut_t), ib = L->idx_lut.size() * sizeof(lut_t);
        std::memcpy(image.data(), L->val_lut.data(), vb);
        std::memcpy(image.data() + vb, L->idx_lut.data(), ib);
        std::memcpy(image.data() + ((vb + ib + 15) & ~(size_t)15), L->codebook.data(), L->codebook.size() * 4);
    }
    Sec secs[6] = {
        {L->records.data(), L->records.size() * 8, 0},
        {L->meta.data(), L->meta.size() * sizeof(cl_chunk_meta), 0},
        {L->block_ptr.data(), L->block_ptr.size() * 4, 0},
        {L->panel_chunk.data(), L->panel_chunk.size() * 4, 0},
        {image.data(), image.size(), 0},
        {L->block_chunk.data(), L->block_chunk.size() * 4, 0},
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
    size_t lds_for(const cl_layer *L, int bt) const { return fixed + ((size_t)L->desc.block_h + xcap_for(bt)) * 4 * bt; }
};

int32_t plan_sparse(const cl_layer *L, int batch, size_t max_lds, SparsePlan &P)
{
    P.fixed = table_image_bytes(L->val_lut_bits, L->idx_lut_bits, 1 << L->desc.weight_bits);
    P.xwant = (int)std::min<int64_t>(L->desc.K, (1 + 2 * kSparseChunksPerWave) * (int64_t)L->desc.block_w);
    // largest power-of-two batch tile (<= 16) that fits; prefer to stay under 64 KiB
    size_t budget = std::min<size_t>(max_lds, 64 * 1024);
    if (P.lds_for(L, 1) > budget) budget = max_lds;
    if (P.lds_for(L, 1) > budget) return fail(CL_EUNSUPPORTED, "block_h %d needs more LDS than a workgroup has", L->desc.block_h);
    P.bt_max = 16;
    while (P.bt_max > 1 && (P.lds_for(L, P.bt_max) > budget || P.bt_max / 2 >= batch)) P.bt_max >>= 1;
    P.wg_per_panel = (int)((L->max_panel_chunks + kWaves * kSparseChunksPerWave - 1) / (kWaves * kSparseChunksPerWave));
    P.part_bytes = (size_t)L->n_panels * P.wg_per_panel * L->desc.block_h * P.bt_max * sizeof(float);
    return CL_OK;
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

bool mfma_capable(const cl_layer *L) { return L->desc.block_h <= kTile && L->desc.block_w <= kTile; }

// Image tile, padded column count and split of the block rows for `ncols` columns and
// `panels` block rows, from a small model of the kernel with measured constants
// (cycles per workgroup: 12 k to start; per block 5 k of decoding and bookkeeping plus
// 4.1 k of multiplies per 32 columns of the tile - 1.5 k on the bf16 matrix cores;
// workgroups run in rounds of one per CU).  The model is coarse, so a candidate must win by a sixteenth to replace a
// narrower one.
void mfma_shape(const cl_layer *L, int panels, int ncols, int cus, bool bf16, int &nq, int &np, int &splits)
{
    cus = std::max(1, cus);
    nq = 0;
    int64_t best = -1;
    for (int q : {1, 2, 4, 8}) {
        const int w = 32 * q;
        const int cols = (ncols + w - 1) / w * w;
        const int64_t tiles = (int64_t)panels * (cols / w);
        // the split that fills the CUs, or any smaller one that needs fewer rounds
        const int sp_max = (int)std::max<int64_t>(1, std::min<int64_t>(L->nbw, (cus + tiles - 1) / tiles));
        for (int sp = 1; sp <= sp_max; ++sp) {
            const int64_t rounds = (tiles * sp + cus - 1) / cus;
            const int64_t blocks = (L->nbw + sp - 1) / sp;
            const int64_t t = rounds * (12000 + blocks * (5000 + (bf16 ? 1500 : 4100) * q));
            if (best < 0 || (q == nq ? t < best : t + t / 16 < best)) {
                best = t;
                nq = q;
                np = cols;
                splits = sp;
            }
        }
    }
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
                       const float *xt, float *part, hipStream_t st)
{
    static LdsLimit seen;
    if (int32_t rc = ensure_lds((const void *)fc_mfma_kernel<NQ>, lds, seen)) return rc;
    hipLaunchKernelGGL(fc_mfma_kernel<NQ>, dim3((unsigned)(panels * splits * (np / MfmaShape<NQ>::kImages))),
                       dim3(MfmaShape<NQ>::kThreads), lds, st, D, xt, part, splits, np, panels_per_x, x_stride);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

template <int NQ>
int32_t launch_bf16_as(const LayerDev &D, int panels, int splits, int np, int panels_per_x, size_t x_stride, size_t lds,
                       const uint16_t *xb, size_t plane_elems, float *part, hipStream_t st)
{
    static LdsLimit seen;
    if (int32_t rc = ensure_lds((const void *)fc_mfma_bf16_kernel<NQ>, lds, seen)) return rc;
    hipLaunchKernelGGL(fc_mfma_bf16_kernel<NQ>, dim3((unsigned)(panels * splits * (np / Bf16Shape<NQ>::kImages))),
                       dim3(Bf16Shape<NQ>::kThreads), lds, st, D, xb, part, splits, np, plane_elems, panels_per_x, x_stride);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

// panels block rows in one launch; each run of panels_per_x of them multiplies an
// activation matrix of its own, x_bytes after the one before
int32_t launch_mfma(const cl_layer *L, const LayerDev &D, bool bf16, int nq, int panels, int splits, int np, int panels_per_x,
                    size_t x_bytes, size_t lds, const void *xt, float *part, hipStream_t st)
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
        case 1: return launch_mfma_as<1>(D, panels, splits, np, panels_per_x, x_stride, lds, (const float *)xt, part, st);
        case 2: return launch_mfma_as<2>(D, panels, splits, np, panels_per_x, x_stride, lds, (const float *)xt, part, st);
        case 4: return launch_mfma_as<4>(D, panels, splits, np, panels_per_x, x_stride, lds, (const float *)xt, part, st);
        case 8: return launch_mfma_as<8>(D, panels, splits, np, panels_per_x, x_stride, lds, (const float *)xt, part, st);
        }
    }
    return fail(CL_EINVAL, "internal: no dense-tile kernel for %d accumulators", nq);
}

// CL_PATH_AUTO: the sparse path up to kAutoSparseBatch images, the dense-tile path
// above when the blocks fit a tile.  Measured on the AlexNet-shaped stack (fc6 / fc7 /
// fc8, ms): sparse 0.037 / 0.024 / 0.019 at 4 images and 0.061 / 0.038 / 0.028 at 5-8
// (its batch tile is a power of two); dense tiles of 32 images 0.048 / 0.028 / 0.021.
constexpr int kAutoSparseBatch = 4;

int resolve_path(const cl_layer *L, int batch, int path)
{
    if (path != CL_PATH_AUTO) return path;
    return (batch > kAutoSparseBatch && mfma_capable(L)) ? CL_PATH_MFMA_F32 : CL_PATH_SPARSE;
}

bool is_mfma(int path) { return path == CL_PATH_MFMA_F32 || path == CL_PATH_MFMA_BF16; }

}  // namespace

extern "C" int32_t cl_fc_workspace_bytes(const cl_layer *L, int32_t batch, int32_t path, size_t *out)
{
    if (!L || !out) return fail(CL_EINVAL, "null argument");
    if (batch < 1) return fail(CL_EINVAL, "batch must be positive");
    if (path < CL_PATH_AUTO || path > CL_PATH_MFMA_BF16) return fail(CL_EINVAL, "unknown path %d", path);
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    const int chosen = resolve_path(L, batch, path);
    if (is_mfma(chosen)) {
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

static int32_t forward_sparse(const cl_layer *L, const LayerDev &D, const DeviceLimits &dl, const float *d_X,
                              const float *d_bias, float *d_Y, int batch, int relu, float *part, hipStream_t st)
{
    SparsePlan P;
    if (int32_t rc = plan_sparse(L, batch, dl.max_lds, P)) return rc;
    const int M = L->desc.M, K = L->desc.K;
    const dim3 grid((unsigned)(L->n_panels * P.wg_per_panel));
    for (int b0 = 0; b0 < batch;) {
        int bt = P.bt_max;
        while (bt > batch - b0) bt >>= 1;
        const float *x = d_X + (size_t)b0 * K;
        float *y = d_Y + (size_t)b0 * M;
        if (L->n_chunks > 0) {
            const size_t lds = P.lds_for(L, bt);
            const int xcap = P.xcap_for(bt);
            if (b0 == 0) timing_begin(st);      // benchmarks time the first main-kernel launch of a call
#define CL_LAUNCH_SPARSE(BTV)                                                                                      \
    do {                                                                                                           \
        if (lds > 64 * 1024)                                                                                       \
            HIP_TRY(hipFuncSetAttribute((const void *)fc_sparse_kernel<BTV>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
        hipLaunchKernelGGL(fc_sparse_kernel<BTV>, grid, dim3(kThreads), lds, st, D, x, part, P.wg_per_panel, xcap); \
    } while (0)
            switch (bt) {
            case 16: CL_LAUNCH_SPARSE(16); break;
            case 8: CL_LAUNCH_SPARSE(8); break;
            case 4: CL_LAUNCH_SPARSE(4); break;
            case 2: CL_LAUNCH_SPARSE(2); break;
            default: CL_LAUNCH_SPARSE(1); break;
            }
#undef CL_LAUNCH_SPARSE
            HIP_TRY(hipGetLastError());
            if (b0 == 0) timing_end(st, 1);
        }
        hipLaunchKernelGGL(fc_reduce_kernel, dim3((unsigned)(L->n_panels * bt)), dim3(kRedThreads), 0, st,
                           D, part, d_bias, y, bt, bt, P.wg_per_panel, relu);
        HIP_TRY(hipGetLastError());
        b0 += bt;
    }
    return CL_OK;
}

static int32_t forward_mfma(const cl_layer *L, const LayerDev &D, const DeviceLimits &dl, bool bf16, const float *d_X,
                            const float *d_bias, float *d_Y, int batch, int relu, char *ws, hipStream_t st)
{
    MfmaPlan P;
    if (int32_t rc = plan_mfma(L, batch, bf16, dl, P)) return rc;
    const int K = L->desc.K;
    float *part = (float *)(ws + P.xt_bytes);
    if (bf16) {
        hipLaunchKernelGGL(split_pad_kernel, dim3((unsigned)(L->nbw * 8), (unsigned)((P.Bp + 63) / 64)), dim3(256), 0, st,
                           d_X, (uint16_t *)ws, batch, K, P.Bp, L->desc.block_w, xb_plane_elems(L, P.Bp));
    } else {
        const int rows = L->nbw * kTile;
        hipLaunchKernelGGL(transpose_pad_kernel, dim3((unsigned)(rows / 32), (unsigned)(P.Bp / 32)), dim3(256), 0, st,
                           d_X, (float *)ws, batch, K, P.Bp, L->desc.block_w, rows);
    }
    HIP_TRY(hipGetLastError());
    timing_begin(st);
    if (int32_t rc = launch_mfma(L, D, bf16, P.nq, L->n_panels, P.splits, P.Bp, L->n_panels, 0, P.lds, ws, part, st)) return rc;
    timing_end(st, 1);
    const int ct = reduce_col_tile(L->n_panels, batch);
    hipLaunchKernelGGL(mfma_reduce_kernel, dim3((unsigned)(L->n_panels * ((batch + ct - 1) / ct))), dim3(256), 0, st,
                       D, part, d_bias, d_Y, batch, P.Bp, P.splits, relu, 0, ct);
    HIP_TRY(hipGetLastError());
    return CL_OK;
}

extern "C" int32_t cl_compressed_fc_forward(const cl_layer *L, const float *d_X, const float *d_bias,
                                            float *d_Y, int32_t batch, int32_t relu, int32_t path,
                                            void *d_workspace, size_t workspace_bytes, void *stream)
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
    const int chosen = resolve_path(L, batch, path);
    if (is_mfma(chosen))
        rc = forward_mfma(L, D, dl, chosen == CL_PATH_MFMA_BF16, d_X, d_bias, d_Y, batch, relu, (char *)d_workspace, (hipStream_t)stream);
    else
        rc = forward_sparse(L, D, dl, d_X, d_bias, d_Y, batch, relu, (float *)d_workspace, (hipStream_t)stream);
    if (rc == CL_OK) clear_error();
    return rc;
}

// ------------------------------------------------------------------------- //
// fixed-function layers of a whole network (Table IV: pool, norm)
// ------------------------------------------------------------------------- //
namespace cl {

__global__ __launch_bounds__(256) void maxpool_kernel(const float *__restrict__ X, float *Y, int64_t n_out, int H, int W,
                                                      int P, int Q, int size, int stride)
{
    for (int64_t o = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; o < n_out; o += (int64_t)gridDim.x * blockDim.x) {
        const int q = (int)(o % Q), p = (int)((o / Q) % P);
        const int64_t bc = o / ((int64_t)P * Q);
        const float *x = X + (bc * H + (int64_t)p * stride) * W + (int64_t)q * stride;
        float m = x[0];
        for (int r = 0; r < size; ++r)
            for (int s = 0; s < size; ++s) m = fmaxf(m, x[(int64_t)r * W + s]);
        Y[o] = m;
    }
}

// One thread per (image, pixel) walks the channels with a sliding sum of squares.
__global__ __launch_bounds__(256) void lrn_kernel(const float *__restrict__ X, float *Y, int B, int C, int64_t hw, int n,
                                                  float alpha_over_n, float beta, float k)
{
    const int half = n / 2;
    for (int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; t < (int64_t)B * hw; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t b = t / hw, i = t - b * hw;
        const float *x = X + b * C * hw + i;
        float *y = Y + b * C * hw + i;
        for (int c = 0; c < C; ++c) {
            float ss = 0.0f;
            for (int cc = max(0, c - half); cc <= min(C - 1, c + half); ++cc) {
                const float v = x[(int64_t)cc * hw];
                ss += v * v;
            }
            y[(int64_t)c * hw] = x[(int64_t)c * hw] * powf(k + alpha_over_n * ss, -beta);
        }
    }
}

}  // namespace cl

extern "C" int32_t cl_maxpool_forward(const float *d_X, float *d_Y, int32_t batch, int32_t C, int32_t H, int32_t W,
                                      int32_t size, int32_t stride, void *stream)
{
    if (!d_X || !d_Y) return fail(CL_EINVAL, "null pointer");
    if (batch < 1 || C < 1 || size < 1 || stride < 1 || H < size || W < size) return fail(CL_EINVAL, "bad pooling geometry");
    const int P = (H - size) / stride + 1, Q = (W - size) / stride + 1;
    const int64_t n_out = (int64_t)batch * C * P * Q;
    hipLaunchKernelGGL(maxpool_kernel, dim3((unsigned)std::min<int64_t>((n_out + 255) / 256, 65536)), dim3(256), 0, (hipStream_t)stream,
                       d_X, d_Y, n_out, H, W, P, Q, size, stride);
    HIP_TRY(hipGetLastError());
    clear_error();
    return CL_OK;
}

extern "C" int32_t cl_lrn_forward(const float *d_X, float *d_Y, int32_t batch, int32_t C, int32_t H, int32_t W,
                                  int32_t n, float alpha, float beta, float k, void *stream)
{
    if (!d_X || !d_Y) return fail(CL_EINVAL, "null pointer");
    if (batch < 1 || C < 1 || H < 1 || W < 1 || n < 1 || !(n & 1)) return fail(CL_EINVAL, "bad normalisation geometry");
    const int64_t hw = (int64_t)H * W, threads = (int64_t)batch * hw;
    hipLaunchKernelGGL(lrn_kernel, dim3((unsigned)std::min<int64_t>((threads + 255) / 256, 65536)), dim3(256), 0, (hipStream_t)stream,
                       d_X, d_Y, batch, C, hw, n, alpha / (float)n, beta, k);
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
    size_t lds = 0, xt_bytes = 0, part_bytes = 0;
};

int32_t plan_conv(const cl_layer *L, const cl_conv_desc *cv, int batch, bool bf16, const DeviceLimits &dl, ConvPlan &P)
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
    if (L->desc.M != cv->out_channels || L->desc.K != g.Cg * g.R * g.S)
        return fail(CL_EINVAL, "layer is %d x %d, the convolution needs %d x %d", L->desc.M, L->desc.K, cv->out_channels, g.Cg * g.R * g.S);
    if (!mfma_capable(L)) return fail(CL_EUNSUPPORTED, "the convolution path needs blocks of at most %d x %d", kTile, kTile);
    P.OCg = cv->out_channels / cv->groups;
    if (cv->groups > 1 && P.OCg % L->desc.block_h) return fail(CL_EUNSUPPORTED, "block_h %d must divide the %d filters of a group", L->desc.block_h, P.OCg);
    P.panels_per_group = (P.OCg + L->desc.block_h - 1) / L->desc.block_h;
    const size_t per_image = (size_t)cv->groups * xt_rows(L) * g.P * g.Q * sizeof(float);
    P.imgs = (int)std::max<size_t>(1, std::min<size_t>((size_t)batch, kConvXtCap / per_image));
    P.lds = mfma_lds_bytes(L, bf16);
    if (P.lds > dl.max_lds) return fail(CL_EUNSUPPORTED, "the convolution path needs %zu bytes of LDS", P.lds);
    // workspace for the larger of a full image group and the last, smaller one
    P.xt_bytes = P.part_bytes = 0;
    for (int imgs : {P.imgs, batch % P.imgs}) {
        if (imgs == 0) continue;
        int nq, np, splits;
        mfma_shape(L, L->n_panels, imgs * g.P * g.Q, dl.cus, bf16, nq, np, splits);
        P.xt_bytes = std::max(P.xt_bytes, (size_t)cv->groups * xt_bytes_for(L, np, bf16));
        P.part_bytes = std::max(P.part_bytes, (size_t)L->n_panels * splits * np * L->desc.block_h * sizeof(float));
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
    *out = P.xt_bytes + P.part_bytes;
    return CL_OK;
}

extern "C" int32_t cl_compressed_conv_forward(const cl_layer *L, const cl_conv_desc *cv, const float *d_X,
                                              const float *d_bias, float *d_Y, int32_t batch, int32_t relu,
                                              int32_t path, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (int32_t rc = require_device(L)) return rc;
    if (!d_X || !d_Y) return fail(CL_EINVAL, "null activation pointer");
    size_t need = 0;
    if (int32_t rc = cl_conv_workspace_bytes(L, cv, batch, path, &need)) return rc;
    if (workspace_bytes < need || !d_workspace) return fail(CL_EINVAL, "workspace too small: %zu < %zu", workspace_bytes, need);
    if ((uintptr_t)d_workspace % 256) return fail(CL_EINVAL, "workspace must be 256-byte aligned");
    DeviceLimits dl;
    if (int32_t rc = device_limits(dl)) return rc;
    const bool bf16 = path == CL_PATH_MFMA_BF16;
    ConvPlan P;
    if (int32_t rc = plan_conv(L, cv, batch, bf16, dl, P)) return rc;
    hipStream_t st = (hipStream_t)stream;
    const LayerDev D = make_dev(L);
    const ConvGeom &g = P.cg;
    const int pq = g.P * g.Q, M = L->desc.M, K = L->desc.K;
    void *xt = d_workspace;
    float *part = (float *)((char *)d_workspace + P.xt_bytes);
    bool timed = false;
    for (int b0 = 0; b0 < batch; b0 += P.imgs) {
        const int nb = std::min(P.imgs, batch - b0);
        const int ncols = nb * pq;
        int nq, Np, splits;
        mfma_shape(L, L->n_panels, ncols, dl.cus, bf16, nq, Np, splits);
        const float *x = d_X + (size_t)b0 * g.C * g.H * g.W;
        float *y = d_Y + (size_t)b0 * M * pq;
        // all filter groups in one launch of each kernel: group grp has its column matrix
        // at xt + grp * x_bytes and multiplies block rows grp * panels_per_group onwards
        const size_t x_bytes = xt_bytes_for(L, Np, bf16);
        const unsigned groups = (unsigned)cv->groups;
        if (bf16)
            hipLaunchKernelGGL(im2col_split_kernel, dim3((unsigned)std::min((Np + 63) / 64, 4096), (unsigned)(L->nbw * 8), groups), dim3(256), 0, st,
                               x, (uint16_t *)xt, g, x_bytes / sizeof(uint16_t), ncols, Np, L->desc.block_w, K, xb_plane_elems(L, Np));
        else
            hipLaunchKernelGGL(im2col_pad_kernel, dim3((unsigned)std::min((Np / 4 + 255) / 256, 1024), (unsigned)(L->nbw * kTile), groups), dim3(256), 0, st,
                               x, (float *)xt, g, x_bytes / sizeof(float), ncols, Np, L->desc.block_w, K);
        HIP_TRY(hipGetLastError());
        if (!timed) timing_begin(st);
        if (int32_t rc = launch_mfma(L, D, bf16, nq, L->n_panels, splits, Np, P.panels_per_group, x_bytes, P.lds, xt, part, st)) return rc;
        if (!timed) { timing_end(st, 1); timed = true; }
        const int ct = reduce_col_tile(L->n_panels, ncols);
        hipLaunchKernelGGL(mfma_reduce_kernel, dim3((unsigned)(L->n_panels * ((ncols + ct - 1) / ct))), dim3(256), 0, st,
                           D, part, d_bias, y, ncols, Np, splits, relu, pq, ct);
        HIP_TRY(hipGetLastError());
    }
    clear_error();
    return CL_OK;
}
