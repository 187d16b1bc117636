// Wavefront primitives, lane records, the decoding and placement passes (Algorithm 2 steps 5-9), block geometry and the LDS image of the decode tables.
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

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

// and the store
template <int W> __device__ __forceinline__ void store_floats(float *p, const float *src)
{
    typedef float vec_t __attribute__((ext_vector_type(W)));
    vec_t v;
#pragma unroll
    for (int i = 0; i < W; ++i) v[i] = src[i];
    *(vec_t *)p = v;
}

template <> __device__ __forceinline__ void store_floats<1>(float *p, const float *src) { *p = src[0]; }

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

// The same walk over a record's entries for callers that look a value up per entry and
// then store it: the entries are taken four at a time, the four look-ups (made in every
// lane, value index 0 for entries a lane does not have) go out together and are waited
// for once, then put(position, looked-up value) is called for the lane's own entries.
template <int J, class Look, class Put>
__device__ __forceinline__ void place_from(const Symbols &y, uint32_t pos, Look &look, Put &put)
{
    if constexpr (J < kMaxEntries) {
        if ((uint32_t)J >= y.nmax) return;                                  // uniform, once per four entries
        constexpr int G = kMaxEntries - J < 4 ? kMaxEntries - J : 4;
        uint32_t at[G];
        decltype(look(0u)) w[G];
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const uint32_t z = (y.z[J / 4] >> (8 * u)) & 0xffu, v = (y.v[J / 4] >> (8 * u)) & 0xffu;
            pos += z + 1u;
            at[u] = pos;
            w[u] = look(v);
        }
#pragma unroll
        for (int u = 0; u < G; ++u)
            if ((uint32_t)(J + u) < y.n) put(at[u], w[u]);
        place_from<J + G>(y, pos, look, put);
    }
}

template <class Look, class Put>
__device__ __forceinline__ void place_entries(const Symbols &y, uint32_t sum, Look look, Put put)
{
    place_from<0>(y, sum - 1u, look, put);
}

// The walk for callers that fetch something per entry and then work on it in order: the
// entries are taken G at a time, fetch(u, v, position) is called for the G of them first (in
// every lane, value index 0 and a position one further for entries a lane does not have),
// so that what it loads is in flight together and waited for once; then use(u) for the
// lane's own entries, in order.  fetch and use share their storage through the slot number
// u < G.  Entries past the wavefront's longest record are skipped.
template <int G, int J, class Fetch, class Use>
__device__ __forceinline__ void groups_from(const Symbols &y, uint32_t pos, Fetch &fetch, Use &use)
{
    if constexpr (J < kMaxEntries) {
        if ((uint32_t)J >= y.nmax) return;                                  // uniform, once per group
        constexpr int N = kMaxEntries - J < G ? kMaxEntries - J : G;
#pragma unroll
        for (int u = 0; u < N; ++u) {
            if ((uint32_t)(J + u) < y.nmax) {                               // uniform
                const uint32_t z = (y.z[(J + u) / 4] >> (8 * ((J + u) % 4))) & 0xffu, v = (y.v[(J + u) / 4] >> (8 * ((J + u) % 4))) & 0xffu;
                pos += z + 1u;
                fetch(u, v, pos);
            }
        }
#pragma unroll
        for (int u = 0; u < N; ++u)
            if ((uint32_t)(J + u) < y.n) use(u);
        groups_from<G, J + N>(y, pos, fetch, use);
    }
}

template <int G, class Fetch, class Use>
__device__ __forceinline__ void for_each_entry_grouped(const Symbols &y, uint32_t sum, Fetch fetch, Use use)
{
    groups_from<G, 0>(y, sum - 1u, fetch, use);
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
