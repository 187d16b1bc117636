// Large batches on the vector ALUs: the sparse product of Algorithm 2 step 12 as written -
// one multiply-add per surviving weight and image, no dense tile - with the images across
// the lanes (lane l: images IPL l .. IPL l + IPL - 1 of a tile of 64 IPL images, IPL = 1, 2
// or 4).  wide_expand_kernel, wide_mul_kernel and the finishing kernel.
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

constexpr int kWideWaves = 16;
constexpr int kWideThreads = kWideWaves * 64;
constexpr int kHalf = 64;                                               // columns per slab
constexpr int kSlabRowsPerWave = kHalf / kWideWaves;                    // rows of a slab each wavefront copies

// IPL consecutive floats from LDS / to LDS / from global memory with one access.
template <int IPL> struct WideVec {
    typedef float type __attribute__((ext_vector_type(IPL)));
};
template <> struct WideVec<1> {
    typedef float type;
};

// ------------------------------------------------------------------------- //
// Two launches: decode to an entry list, then multiply
// ------------------------------------------------------------------------- //
// wide_expand_kernel decodes the whole layer once per call (Algorithm 2 steps 5-9, one
// wavefront per chunk as in decode_kernel) into a list in global memory: a block's
// surviving weights - the padding entries dropped - in the order the multiplying kernel
// takes them: first those in the block's columns 0-63, then those in columns 64-127,
// each half row by row.  Where a chunk's entries go in that order does not depend on the
// activations: the layer carries, per chunk, the list position of its first surviving
// weight of each half (chunk_half), and, per block and half, where each group of eight
// rows starts (group_ptr), both counted when the layer was loaded.  An entry is one word:
// the value index (bits 16-23), the column within the half (bits 8-13) and IPL times the
// row within its group of eight (bits 0-7: the offset of the row's sums among the
// multiplying wavefront's sum registers).
// wide_mul_kernel then holds no decode tables, decodes nothing and waits for no decoder:
// sixteen wavefronts multiply, each owning the eight rows of one group, the weights looked
// up in the codebook (Algorithm 2 step 8) 64 entries at a time, and every image tile of a
// large batch reads the same list.
typedef uint32_t WideEntry;
constexpr int kMulRows = kTile / kWideWaves;            // rows of a block row per wavefront: a group
constexpr int kGroupPtrs = 2 * (kWideWaves + 1);        // group_ptr words per block

// (One launch can decode several layers - those of a stack that take this path - each into
// its own list: workgroups wg0[i] .. wg0[i + 1] - 1 belong to job i.)
constexpr int kExpandJobs = 4;
struct ExpandJobs {
    LayerDev L[kExpandJobs];
    WideEntry *ent[kExpandJobs];
    uint32_t wg0[kExpandJobs + 1];
    uint32_t ipl;                   // images per lane of the multiplying kernel: the row offsets count its sum registers
    // The same launch can lay out the activations of the first layer (what transpose_pad_kernel
    // does: XT rows x Bp from X B x K): its first t_wgs workgroups do that, two 32 x 32 tiles
    // each, and are through while the decoding workgroups wait for their records.
    const float *X;
    float *XT;
    int B, K, Bp, bw, rows;
    uint32_t t_wgs;
};

__global__ __launch_bounds__(kThreads) void wide_expand_kernel(ExpandJobs jobs)
{
    if (blockIdx.x < jobs.t_wgs) {
        __shared__ float t[2][32][33];
        const int half = (int)(threadIdx.x >> 8), tid = (int)(threadIdx.x & 255);
        const int row_tiles = jobs.rows / 32, tile = (int)blockIdx.x * 2 + half;
        const bool real = tile < row_tiles * (jobs.Bp / 32);
        const int r0 = (tile % row_tiles) * 32, b0 = (tile / row_tiles) * 32;
        const int tx = tid & 31, ty = tid >> 5;       // 32 x 8
        if (real)
            for (int i = ty; i < 32; i += 8) {
                const int b = b0 + i, k = xt_row_to_k(r0 + tx, jobs.bw, jobs.K);
                t[half][i][tx] = (b < jobs.B && k >= 0) ? jobs.X[(size_t)b * jobs.K + k] : 0.0f;
            }
        __syncthreads();
        if (real)
            for (int i = ty; i < 32; i += 8) jobs.XT[(size_t)(r0 + i) * jobs.Bp + b0 + tx] = t[half][tx][i];
        return;
    }
    int job = 0;
#pragma unroll
    for (int i = 1; i < kExpandJobs; ++i)
        if (blockIdx.x >= jobs.wg0[i]) job = i;
    const LayerDev &L = jobs.L[job];
    WideEntry *ent = jobs.ent[job];
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const uint32_t c = (blockIdx.x - jobs.wg0[job]) * kWaves + (uint32_t)wave;
    const bool have = c < L.n_chunks;
    ChunkHead h{};
    LaneRecord rec{};
    uint32_t base0 = 0, base1 = 0;
    if (have) {
        h = load_head(L, c);
        rec = load_record(L, h, lane);
        base0 = L.chunk_half[2 * (size_t)c];
        base1 = L.chunk_half[2 * (size_t)c + 1];
    }
    store_tables(s, L, fetch_tables(L));
    __syncthreads();
    if (!have) return;
    const BlockGeom g = block_geom(L, h.m.blk);
    const Symbols y = decode_record(rec, s.T);
    const LaneStart st = lane_starts(y, h.m.pos0);
    // the lane's surviving weights per half, then where its first of each half goes
    uint32_t mine = 0;
    for_each_entry(y, st.sum, [&](uint32_t, uint32_t v, uint32_t, uint32_t pos) {
        uint32_t r, cc;
        split_pos(pos, g, r, cc);
        if (v != 0u) mine += cc >= (uint32_t)kHalf ? 0x10000u : 1u;
    });
    const uint32_t excl = wave_incl_scan(mine) - mine;
    uint32_t at0 = base0 + (excl & 0xffffu), at1 = base1 + (excl >> 16);
    for_each_entry(y, st.sum, [&](uint32_t, uint32_t v, uint32_t, uint32_t pos) {
        uint32_t r, cc;
        split_pos(pos, g, r, cc);
        if (v == 0u) return;
        const WideEntry e = (v << 16) | ((cc & (uint32_t)(kHalf - 1)) << 8) | ((r & (uint32_t)(kMulRows - 1)) * jobs.ipl);
        if (cc >= (uint32_t)kHalf) ent[at1++] = e;
        else ent[at0++] = e;
    });
}

// The multiply-add of up to 64 entries, one per lane of (entry word, weight) - lanes past
// the last entry holding a copy of the last one with weight zero - into the sums of the
// entries' rows: sums[IPL r + q] += w * x[column][IPL lane + q].  The rows differ from entry to entry
// and the sums live in registers, so the register a product is added to is picked at run
// time: the sums sit in v[64:95], the additions run in the vector-register index mode
// with the entry's row offset as the index (destination and addend relative), and
// everything between switching the mode on and off is written out here.  Entries are
// taken four at a time, the activations of the next four requested from LDS (into
// v[96:127], alternating halves) before the products of the present four are formed, so
// that the loads and the arithmetic overlap from one end of the list to the other
// whatever the rows' lengths.
// (X = images per lane, 4, 2 or 1: the slab row is 256 X bytes, the LDS read X floats wide,
// X multiply-adds per entry, the row offset in the entry word X (row mod 8).)
#define WM_RL(i, slot)                                                                       \
    "v_readlane_b32 %[c" #slot "], %[vat], " #i "\n"                                         \
    "v_readlane_b32 %[w" #slot "], %[vw], " #i "\n"
#define WM_AD_4(slot, tmp)                                                                   \
    "s_and_b32 %[" #tmp "], %[c" #slot "], 0x3f00\n"                                         \
    "v_lshl_add_u32 v[" #slot "*4+96], %[" #tmp "], 2, %[base]\n"
#define WM_AD_2(slot, tmp)                                                                   \
    "s_and_b32 %[" #tmp "], %[c" #slot "], 0x3f00\n"                                         \
    "v_lshl_add_u32 v[" #slot "*4+96], %[" #tmp "], 1, %[base]\n"
#define WM_AD_1(slot, tmp)                                                                   \
    "s_and_b32 %[" #tmp "], %[c" #slot "], 0x3f00\n"                                         \
    "v_add_u32 v[" #slot "*4+96], %[" #tmp "], %[base]\n"
#define WM_RD_4(slot) "ds_read_b128 v[" #slot "*4+96:" #slot "*4+99], v[" #slot "*4+96]\n"
#define WM_RD_2(slot) "ds_read_b64 v[" #slot "*4+96:" #slot "*4+97], v[" #slot "*4+96]\n"
#define WM_RD_1(slot) "ds_read_b32 v[" #slot "*4+96], v[" #slot "*4+96]\n"
#define WM_FMA1_4(slot)                                                                      \
    "s_set_gpr_idx_on %[c" #slot "], 0xc\n"                                                  \
    "v_fma_f32 v64, %[w" #slot "], v[" #slot "*4+96], v64\n"                                 \
    "v_fma_f32 v65, %[w" #slot "], v[" #slot "*4+97], v65\n"                                 \
    "v_fma_f32 v66, %[w" #slot "], v[" #slot "*4+98], v66\n"                                 \
    "v_fma_f32 v67, %[w" #slot "], v[" #slot "*4+99], v67\n"
#define WM_FMA1_2(slot)                                                                      \
    "s_set_gpr_idx_on %[c" #slot "], 0xc\n"                                                  \
    "v_fma_f32 v64, %[w" #slot "], v[" #slot "*4+96], v64\n"                                 \
    "v_fma_f32 v65, %[w" #slot "], v[" #slot "*4+97], v65\n"
#define WM_FMA1_1(slot)                                                                      \
    "s_set_gpr_idx_on %[c" #slot "], 0xc\n"                                                  \
    "v_fma_f32 v64, %[w" #slot "], v[" #slot "*4+96], v64\n"
#define WM_LOAD4(X, i0, i1, i2, i3, s0, s1, s2, s3)                                          \
    WM_RL(i0, s0) WM_RL(i1, s1) WM_RL(i2, s2) WM_RL(i3, s3)                                  \
    WM_AD_##X(s0, t) WM_AD_##X(s1, t2) WM_AD_##X(s2, t) WM_AD_##X(s3, t2)                    \
    WM_RD_##X(s0) WM_RD_##X(s1) WM_RD_##X(s2) WM_RD_##X(s3)
#define WM_FMA4(X, s0, s1, s2, s3) WM_FMA1_##X(s0) WM_FMA1_##X(s1) WM_FMA1_##X(s2) WM_FMA1_##X(s3) "s_set_gpr_idx_off\n"
// entries i0 .. i0 + 3 are in flight in slots (a); request i0 + 4 .. i0 + 7 into slots (b), then add (a)
#define WM_STEP(X, prio, n_done, j0, j1, j2, j3, a0, a1, a2, a3, b0, b1, b2, b3)             \
    "s_setprio " #prio "\n"                                                                  \
    WM_LOAD4(X, j0, j1, j2, j3, b0, b1, b2, b3)                                              \
    "s_waitcnt lgkmcnt(4)\n"                                                                 \
    WM_FMA4(X, a0, a1, a2, a3)                                                               \
    "s_cmp_le_u32 %[n], " #n_done "\n"                                                       \
    "s_cbranch_scc1 1f\n"
#define WM_LAST(X, a0, a1, a2, a3)                                                           \
    "s_waitcnt lgkmcnt(0)\n"                                                                 \
    WM_FMA4(X, a0, a1, a2, a3)
// The four wavefronts of a SIMD would otherwise be served oldest first, finish a list one
// after the other, and the last, alone, cannot keep the vector unit busy (one wavefront
// issues an instruction every four to five cycles, of which 7 in 12 are vector
// arithmetic here): each lowers its priority every few steps of its list, so that one
// that is ahead yields to the others and all four advance together.
#define WM_BODY(X)                                                                           \
    WM_LOAD4(X, 0, 1, 2, 3, 0, 1, 2, 3)                                                      \
    WM_STEP(X, 3, 4, 4, 5, 6, 7, 0, 1, 2, 3, 4, 5, 6, 7)                                     \
    WM_STEP(X, 3, 8, 8, 9, 10, 11, 4, 5, 6, 7, 0, 1, 2, 3)                                   \
    WM_STEP(X, 3, 12, 12, 13, 14, 15, 0, 1, 2, 3, 4, 5, 6, 7)                                \
    WM_STEP(X, 2, 16, 16, 17, 18, 19, 4, 5, 6, 7, 0, 1, 2, 3)                                \
    WM_STEP(X, 2, 20, 20, 21, 22, 23, 0, 1, 2, 3, 4, 5, 6, 7)                                \
    WM_STEP(X, 2, 24, 24, 25, 26, 27, 4, 5, 6, 7, 0, 1, 2, 3)                                \
    WM_STEP(X, 1, 28, 28, 29, 30, 31, 0, 1, 2, 3, 4, 5, 6, 7)                                \
    WM_STEP(X, 1, 32, 32, 33, 34, 35, 4, 5, 6, 7, 0, 1, 2, 3)                                \
    WM_STEP(X, 1, 36, 36, 37, 38, 39, 0, 1, 2, 3, 4, 5, 6, 7)                                \
    WM_STEP(X, 0, 40, 40, 41, 42, 43, 4, 5, 6, 7, 0, 1, 2, 3)                                \
    WM_STEP(X, 0, 44, 44, 45, 46, 47, 0, 1, 2, 3, 4, 5, 6, 7)                                \
    WM_STEP(X, 0, 48, 48, 49, 50, 51, 4, 5, 6, 7, 0, 1, 2, 3)                                \
    WM_STEP(X, 0, 52, 52, 53, 54, 55, 0, 1, 2, 3, 4, 5, 6, 7)                                \
    WM_STEP(X, 0, 56, 56, 57, 58, 59, 4, 5, 6, 7, 0, 1, 2, 3)                                \
    WM_STEP(X, 0, 60, 60, 61, 62, 63, 0, 1, 2, 3, 4, 5, 6, 7)                                \
    WM_LAST(X, 4, 5, 6, 7)                                                                   \
    "1:\n"                                                                                   \
    "s_waitcnt lgkmcnt(0)\n"                                                                 \
    "s_setprio 0\n"
#define WM_OPERANDS                                                                                                           \
    : "+{v[64:95]}"(sums), [c0] "=&s"(c0), [c1] "=&s"(c1), [c2] "=&s"(c2), [c3] "=&s"(c3), [c4] "=&s"(c4), [c5] "=&s"(c5),   \
      [c6] "=&s"(c6), [c7] "=&s"(c7), [w0] "=&s"(w0), [w1] "=&s"(w1), [w2] "=&s"(w2), [w3] "=&s"(w3), [w4] "=&s"(w4),         \
      [w5] "=&s"(w5), [w6] "=&s"(w6), [w7] "=&s"(w7), [t] "=&s"(t), [t2] "=&s"(t2)                                            \
    : [vat] "v"(vat), [vw] "v"(vw), [base] "v"(base), [n] "s"(n)                                                              \
    : "memory", "scc", "m0", "v96", "v97", "v98", "v99", "v100", "v101", "v102", "v103", "v104", "v105", "v106", "v107",      \
      "v108", "v109", "v110", "v111", "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121", "v122", \
      "v123", "v124", "v125", "v126", "v127"

typedef float WideSums __attribute__((ext_vector_type(32)));

template <int IPL>
__device__ __forceinline__ void wide_fma_entries(WideSums &sums, uint32_t vat, uint32_t vw, uint32_t base, int n)
{
    uint32_t c0, c1, c2, c3, c4, c5, c6, c7, w0, w1, w2, w3, w4, w5, w6, w7, t, t2;
    if constexpr (IPL == 4) asm volatile(WM_BODY(4) WM_OPERANDS);
    else if constexpr (IPL == 2) asm volatile(WM_BODY(2) WM_OPERANDS);
    else asm volatile(WM_BODY(1) WM_OPERANDS);
}

// Workgroup (block row p, split j of its blocks, image tile nb) of sixteen wavefronts, one
// to a CU.  A phase is half a block: its 64 columns' activations for the 256 images sit
// in one of two 64 KB slabs, every wavefront multiplies its group's entries of that half,
// and meanwhile brings in its four rows of the next phase's slab (registers first, LDS
// after its arithmetic) and the first 64 of its next entries; one barrier ends the phase.
template <int IPL>
__global__ __launch_bounds__(kWideThreads) void wide_mul_kernel(LayerDev L, const float *__restrict__ XT,
                                                                const WideEntry *__restrict__ ent, float *part, int panels,
                                                                int splits, int Bp)
{
    constexpr int kImages = 64 * IPL;
    typedef typename WideVec<IPL>::type vec_t;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    float *slabs = (float *)smem_raw;                                   // [2][kHalf][kImages]
    float *cb = slabs + 2 * kHalf * kImages;                            // [ncode]
    // consecutive workgroups take the splits of one block row: with the usual eight splits the
    // workgroups that share a range of activation rows share a die's L2
    const int j = (int)blockIdx.x % splits, rest = (int)blockIdx.x / splits;
    const int p = rest % panels, nb = rest / panels;
    const int pj = p * splits + j;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const int blk_lo = (int)(((int64_t)L.nbw * j) / splits), blk_hi = (int)(((int64_t)L.nbw * (j + 1)) / splits);
    const uint32_t pb0 = (uint32_t)p * (uint32_t)L.nbw;
    const int nh = L.bw > kHalf ? 2 : 1;
    const int phases = (blk_hi - blk_lo) * nh;

    // A wavefront's share of a slab: rows 4 wave .. 4 wave + 3, four floats per lane and row.  The
    // slab of phase ph starts at row (blk_lo + ph / nh) 128 + (ph % nh) 64 of the activations: a
    // uniform base that moves from phase to phase, and per lane a constant byte offset per row.
    const char *xbase = (const char *)(XT + (size_t)nb * kImages);
    uint32_t xoff[kSlabRowsPerWave];
#pragma unroll
    for (int q = 0; q < kSlabRowsPerWave; ++q) xoff[q] = (uint32_t)((wave * kSlabRowsPerWave + q) * Bp + lane * IPL) * 4u;
    vec_t stage[kSlabRowsPerWave];
    auto slab_fetch = [&](int ph) {
        const char *src = xbase + ((size_t)(blk_lo + ph / nh) * kTile + (size_t)(ph % nh) * kHalf) * (size_t)Bp * 4;
#pragma unroll
        for (int q = 0; q < kSlabRowsPerWave; ++q) stage[q] = *(const vec_t *)(src + xoff[q]);
    };
    auto slab_store = [&](int ph) {
        float *dst = slabs + (size_t)(ph & 1) * kHalf * kImages + (size_t)(wave * kSlabRowsPerWave) * kImages + lane * IPL;
#pragma unroll
        for (int q = 0; q < kSlabRowsPerWave; ++q) *(vec_t *)(dst + q * kImages) = stage[q];
    };
    // The wavefront's part of the list in each phase - its group of rows in that half of that
    // block - for 64 phases at a time, phase ph0 + lane in lane `lane`: fetched ahead of
    // the loop so that no phase starts by waiting for a pointer.
    uint32_t seg_a = 0, seg_e = 0;
    auto segments = [&](int ph0) {
        const int ph = min(ph0 + lane, phases - 1);
        const uint32_t b = pb0 + (uint32_t)(blk_lo + ph / nh);
        const uint32_t *gp = L.group_ptr + ((size_t)b * 2 + (size_t)(ph % nh)) * (kWideWaves + 1) + wave;
        seg_a = gp[0];
        seg_e = gp[1];
    };
    auto segment = [&](int ph, uint32_t &a, uint32_t &e) {
        a = (uint32_t)__builtin_amdgcn_readlane((int)seg_a, ph & 63);
        e = (uint32_t)__builtin_amdgcn_readlane((int)seg_e, ph & 63);
    };
    // up to 64 entries from list position a on, one per lane
    const uint32_t lane4 = (uint32_t)lane * 4u;
    auto window = [&](uint32_t a, uint32_t e) {
        uint32_t v = 0u;
        if ((uint32_t)lane < e - a) v = *(const uint32_t *)((const char *)(ent + a) + lane4);
        return v;
    };
    auto weight_of = [&](uint32_t entry) { return cb[(entry >> 16) & 0xffu]; };

    WideSums sums;
#pragma unroll
    for (int q = 0; q < 32; ++q) sums[q] = 0.0f;
    if (phases > 0) {
        // Requests run two phases ahead of the arithmetic: while phase ph is multiplied, the slab
        // rows and the first 64 entries of phase ph + 1 are in registers or on their way, and
        // those of ph + 2 are requested at the end of ph - after the rows of ph + 1 have gone
        // from their registers into LDS - by each wavefront as it gets there, not by all
        // sixteen at once behind the barrier.
        // (two sets of registers take turns, the loop is written out for an even and an odd phase:
        // handing a set on from phase to phase would make each phase wait for what it has just requested)
        struct Ahead {
            uint32_t a = 0, e = 0;      // the wavefront's part of the list in that phase
            uint32_t ev = 0;            // its first 64 entries, one per lane
            float w = 0.0f;             // and their weights
        } even, odd;
        // The entries are requested behind the compiler's back and waited for by hand (arrived): a
        // wait of the compiler's own would stand at the top of the next phase, where it would stall
        // on what was requested a moment before.
        auto request_entries = [&](int ph, Ahead &x) {
            x = Ahead{};
            if (ph >= phases) return;
            if (ph > 0 && (ph & 63) == 0) segments(ph);
            segment(ph, x.a, x.e);
            if ((uint32_t)lane < x.e - x.a && x.e > x.a) {
                const uint32_t *src = (const uint32_t *)((const char *)(ent + x.a) + lane4);
                asm volatile("global_load_dword %0, %1, off" : "=v"(x.ev) : "v"(src) : "memory");
            }
        };
        auto request = [&](int ph, Ahead &x) {
            request_entries(ph, x);
            if (ph < phases) slab_fetch(ph);
        };
        // (nothing younger than the entries is in flight where this is called, so the wait is for them alone)
        auto arrived = [&](Ahead &x) {
            __builtin_amdgcn_s_waitcnt(0x0F70);                         // vmcnt(0)
            asm volatile("" : "+v"(x.ev) : : "memory");
        };
        auto phase = [&](int ph, Ahead &cur, Ahead &nxt) {
            const uint32_t base = (uint32_t)(uintptr_t)(slabs + (size_t)(ph & 1) * kHalf * kImages) + (uint32_t)lane * (IPL * 4);
            // 64 entries at a time; a second 64 (a group of rows with more than 64 surviving weights
            // in 64 columns) are waited for where they are requested, so that the wait in front of
            // the first counts only what was requested before it
            uint32_t v = cur.ev;
            float w = cur.w;
            for (uint32_t a = cur.a; a < cur.e;) {
                const int n = (int)min(64u, cur.e - a);
                // lanes past the last entry: that entry again with weight zero
                const uint32_t last = (uint32_t)__builtin_amdgcn_readlane((int)v, n - 1);
                const uint32_t vat = lane < n ? v : last, vw = lane < n ? __builtin_bit_cast(uint32_t, w) : 0u;
                wide_fma_entries<IPL>(sums, vat, vw, base, n);
                a += 64u;
                if (a < cur.e) {
                    v = window(a, cur.e);
                    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0)
                    w = weight_of(v);
                }
            }
            if (ph + 1 < phases) slab_store(ph + 1);
            arrived(nxt);
            nxt.w = weight_of(nxt.ev);
            asm volatile("" : "+v"(nxt.w));                             // looked up here, not behind the requests below
            request(ph + 2, cur);
            __syncthreads();
        };
        // what the first phase needs, all requested before anything is waited for: the first slab
        // rows, the pointers, the codebook; then the entries (they need the pointers)
        slab_fetch(0);
        segments(0);
        const float cbv = (int)threadIdx.x < L.ncode ? L.codebook[threadIdx.x] : 0.0f;
        request_entries(0, even);
        if ((int)threadIdx.x < L.ncode) cb[threadIdx.x] = cbv;
        slab_store(0);
        arrived(even);
        request(1, odd);
        __syncthreads();
        even.w = weight_of(even.ev);
        for (int ph = 0; ph < phases; ph += 2) {
            phase(ph, even, odd);
            if (ph + 1 < phases) phase(ph + 1, odd, even);
        }
    }
    // the wavefront's rows of the workgroup's partial tile, part[pj][row][Bp]: a row's images are contiguous
    float *mine = part + ((size_t)pj * kTile + (size_t)wave * kMulRows) * (size_t)Bp + (size_t)nb * kImages + (size_t)lane * IPL;
#pragma unroll
    for (int r = 0; r < kMulRows; ++r) {
        vec_t v;
        if constexpr (IPL == 1) v = sums[r];
        else {
#pragma unroll
            for (int q = 0; q < IPL; ++q) v[q] = sums[r * IPL + q];
        }
        *(vec_t *)(mine + (size_t)r * Bp) = v;
    }
}

// Finishes the wide path: Y = act(sum over the splits of a block row, in a fixed order,
// + bias) (Eq. 1) from part[block row][split][row][Bp].  A workgroup takes 32 rows and 64
// images.  With next_bp == 0 the output is Y[image][row] (turned in LDS so that both the
// reads and the writes run along memory); else it is the transposed activations of a
// following layer, XT[row][next_bp], the images from `batch` up to next_bp written as
// zeros (the padded images of that layout).
constexpr int kWideRedRows = 32, kWideRedImages = 64;

__global__ __launch_bounds__(256) void wide_reduce_kernel(LayerDev L, const float *__restrict__ part, const float *__restrict__ bias,
                                                          float *Y, int batch, int Bp, int splits, int relu, int next_bp)
{
    __shared__ float tile[kWideRedRows][kWideRedImages + 1];
    const int ncol = max(Bp, next_bp);
    const int nit = (ncol + kWideRedImages - 1) / kWideRedImages, nrt = kTile / kWideRedRows;
    const int p = (int)blockIdx.x / (nit * nrt), rem = (int)blockIdx.x - p * nit * nrt;
    const int r0 = (rem / nit) * kWideRedRows, c0 = (rem % nit) * kWideRedImages;
    const int row_id = p * L.bh;
    const int bhp = min(L.bh, L.M - row_id);
    // thread -> (row, four images)
    const int tr = (int)threadIdx.x / 16, tc = ((int)threadIdx.x % 16) * 4;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int r = r0 + tr + 16 * half, c = c0 + tc;
        float4 t = {0.0f, 0.0f, 0.0f, 0.0f};
        if (r < bhp && c < Bp) {
            const float *src = part + ((size_t)p * splits * kTile + r) * (size_t)Bp + c;
            const size_t split_stride = (size_t)kTile * Bp;
            for (int j = 0; j < splits; j += 8) {           // eight loads in flight, added in order
                float4 a[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) a[u] = *(const float4 *)(src + (size_t)(j + u < splits ? j + u : 0) * split_stride);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (j + u < splits) { t.x += a[u].x; t.y += a[u].y; t.z += a[u].z; t.w += a[u].w; }
            }
            const float bv = bias ? bias[row_id + r] : 0.0f;
            t.x += bv; t.y += bv; t.z += bv; t.w += bv;
            if (relu) { t.x = fmaxf(t.x, 0.0f); t.y = fmaxf(t.y, 0.0f); t.z = fmaxf(t.z, 0.0f); t.w = fmaxf(t.w, 0.0f); }
            // images past the batch are padding: zero whatever the bias made of them
            if (c + 0 >= batch) t.x = 0.0f;
            if (c + 1 >= batch) t.y = 0.0f;
            if (c + 2 >= batch) t.z = 0.0f;
            if (c + 3 >= batch) t.w = 0.0f;
        }
        if (next_bp) {
            if (r < bhp && c < next_bp) *(float4 *)(Y + (size_t)(row_id + r) * next_bp + c) = t;
        } else {
            tile[tr + 16 * half][tc + 0] = t.x;
            tile[tr + 16 * half][tc + 1] = t.y;
            tile[tr + 16 * half][tc + 2] = t.z;
            tile[tr + 16 * half][tc + 3] = t.w;
        }
    }
    if (next_bp) return;
    __syncthreads();
    // thread -> (image, four rows): 32 consecutive rows of an image are 128 contiguous bytes of Y
    const int ti = (int)threadIdx.x / 8, t4 = ((int)threadIdx.x % 8) * 4;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int img = c0 + ti + 32 * half;
        if (img >= batch) continue;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = r0 + t4 + u;
            if (r < bhp) Y[(size_t)img * L.M + row_id + r] = tile[t4 + u][ti + 32 * half];
        }
    }
}
