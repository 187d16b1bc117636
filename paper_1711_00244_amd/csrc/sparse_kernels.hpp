// decode_layer kernel and the small-batch path: fused decode + sparse multiply, and its finishing kernel.
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

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
// Where a layer's input comes from when the layer before it ran on this path too and
// its finishing kernel is left out (a stack of layers at one image, where a launch costs
// as much as the work in it): the partial tiles of that layer's
// workgroups, part[block row][slot][image][row], to be added up in slot order, plus its
// bias, through its activation (Eq. 1) - what fc_reduce_kernel would have written as
// X[image][k], taken by each workgroup for the columns of its own slab only.
struct PrevSlots {
    const float *part;              // null: the input is X
    const uint32_t *panel_chunk;    // of the layer before: how many slots each of its block rows filled
    const float *bias;              // of the layer before, or null
    int bh, wg_per_panel, part_b, relu;
};

// Up to this batch tile, and for block rows of up to 256 rows, every wavefront of the small-
// batch kernel has an output tile of its own in LDS and writes each row sum once, with a
// plain store (see fc_sparse_body); above, the workgroup shares one tile through float atomics
// (8 x bh x BT floats would crowd the CU, and those batch sizes belong to the tile kernels).
constexpr int kPrivateTileBT = 8, kPrivateTileRows = 256;
__host__ __device__ constexpr bool private_tiles(int bh, int bt) { return bt <= kPrivateTileBT && bh <= kPrivateTileRows; }

// Where a column's BT images lie in the LDS slab: as 16-byte groups of four, and for BT > 4 the
// groups of a column rotated by the column number.  Lanes that read group g of 64 arbitrary
// columns then spread over all 32 banks; unrotated, a column stride of 32 or 64 bytes would put
// them on half or a quarter of the banks.
template <int BT> __device__ __forceinline__ int x_group(int col, int g)
{
    if constexpr (BT == 8) return (g + (col >> 2)) & 1;
    else if constexpr (BT == 16) return (g + (col >> 1)) & 3;
    else return g;
}

// Inclusive sums over the lanes of a wavefront in segments: a lane with `start` begins a
// segment.  (value, started) pairs combine as (b.started ? b.value : a.value + b.value,
// a.started | b.started), which is associative, so the usual doubling steps apply.
template <int BT>
__device__ __forceinline__ void wave_segmented_sums(float (&v)[BT], bool start)
{
    uint32_t f = start ? 1u : 0u;
#define CL_SEG_STEP(CTRL, ROWS)                                                                              \
    {                                                                                                        \
        const uint32_t tf = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)f, CTRL, ROWS, 0xf, false);        \
        _Pragma("unroll") for (int b = 0; b < BT; ++b)                                                       \
        {                                                                                                    \
            const float tv = __builtin_bit_cast(                                                             \
                float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v[b]), CTRL, ROWS, 0xf, false)); \
            v[b] = f ? v[b] : v[b] + tv;                                                                     \
        }                                                                                                    \
        f |= tf;                                                                                             \
    }
    CL_SEG_STEP(0x111, 0xf)   // row_shr:1
    CL_SEG_STEP(0x112, 0xf)   // row_shr:2
    CL_SEG_STEP(0x114, 0xf)   // row_shr:4
    CL_SEG_STEP(0x118, 0xf)   // row_shr:8
    CL_SEG_STEP(0x142, 0xa)   // row_bcast:15 into rows 1, 3
    CL_SEG_STEP(0x143, 0xc)   // row_bcast:31 into rows 2, 3
#undef CL_SEG_STEP
}

// (wg: the workgroup's number within the layer's share of the grid; nb <= BT: images that X
// holds - the tile's other images are zeros; FOLD: the input may be the partial tiles of the
// layer before - an instantiation of its own, so that the code for it does not weigh on the
// registers of the others)
template <int BT, bool FOLD>
__device__ __forceinline__ void fc_sparse_body(const LayerDev &L, const float *__restrict__ X, float *part, int wg_per_panel,
                                               int xcap, const PrevSlots &prev, uint32_t wg, int nb)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    const int p = (int)(wg / (uint32_t)wg_per_panel), j = (int)(wg % (uint32_t)wg_per_panel);
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
    const bool priv = private_tiles(L.bh, BT);
    const int n_tiles = priv ? kWaves : 1;
    float *ytile = s.extra;                  // [n_tiles][BT][bh]
    float *xs = ytile + (size_t)n_tiles * L.bh * BT;   // [xcap][BT]: a column's BT images side by side, one LDS read per entry
    // activation columns of the blocks this workgroup's chunks belong to
    const uint32_t pb0 = (uint32_t)p * (uint32_t)L.nbw;
    const uint32_t c_last = min(pc1, my0 + (uint32_t)(kWaves * kSparseChunksPerWave)) - 1u;
    const int col_a = (int)(L.meta[my0].blk - pb0) * L.bw;
    const int col_b = min(L.K, (int)(L.meta[c_last].blk - pb0 + 1u) * L.bw);
    const int width = col_b - col_a;
    const bool slab = width <= xcap;
    if (FOLD && slab && prev.part) {
        // (the host takes this form only for layers whose every workgroup has a slab)
        constexpr uint32_t kPerWg = kWaves * kSparseChunksPerWave;
        for (int t = threadIdx.x; t < width; t += blockDim.x) {
            const int k = col_a + t, pp = k / prev.bh, r = k - pp * prev.bh;
            const int active = (int)((prev.panel_chunk[pp + 1] - prev.panel_chunk[pp] + kPerWg - 1) / kPerWg);
            const float *src = prev.part + (size_t)pp * prev.wg_per_panel * prev.part_b * prev.bh + r;
            const size_t step = (size_t)prev.part_b * prev.bh;
            const float bv = prev.bias ? prev.bias[k] : 0.0f;
#pragma unroll
            for (int b = 0; b < BT; ++b) {
                float acc = 0.0f;
                for (int j = 0; j < active; j += 12) {      // twelve loads in flight, added in slot order
                    float a[12];
#pragma unroll
                    for (int u = 0; u < 12; ++u) a[u] = src[(size_t)(j + u < active ? j + u : j) * step + (size_t)b * prev.bh];
#pragma unroll
                    for (int u = 0; u < 12; ++u)
                        if (j + u < active) acc += a[u];
                }
                acc += bv;
                xs[t * BT + b] = prev.relu ? fmaxf(acc, 0.0f) : acc;
            }
        }
    } else if (slab && BT < 4) {
#pragma unroll
        for (int b = 0; b < BT; ++b)
            for (int t = threadIdx.x; t < width; t += blockDim.x) xs[t * BT + b] = b < nb ? X[(size_t)b * L.K + col_a + t] : 0.0f;
    } else if (slab) {
        // a column's images are requested together and stored together
        for (int t = threadIdx.x; t < width; t += blockDim.x) {
            float v[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) v[b] = b < nb ? X[(size_t)b * L.K + col_a + t] : 0.0f;
            constexpr int kW = BT < 4 ? BT : 4;
#pragma unroll
            for (int q = 0; q < BT / kW; ++q) store_floats<kW>(xs + t * BT + x_group<BT>(t, q) * kW, v + q * kW);
        }
    }
    // (16 bytes at a time, and four outputs per thread at the end, pay from four images on -
    // measured; below, they cost a microsecond of a step)
    if (BT >= 4) {
        const int n = n_tiles * L.bh * BT;          // a multiple of 4
        float4 *z4 = (float4 *)ytile;
        for (int t = threadIdx.x; t < n / 4; t += blockDim.x) z4[t] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    } else {
        for (int t = threadIdx.x; t < n_tiles * L.bh * BT; t += blockDim.x) ytile[t] = 0.0f;
    }
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
        auto entries_shared = [&](auto load_x, auto split) {
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
        // The same into the wavefront's own tile, without atomics (an LDS float atomic costs about
        // three cycles per lane here: half of the kernel at four images).  The chunk's entries
        // run row by row across the lanes, so a row's terms sit in one lane or in a run of
        // neighbouring lanes: a row that begins and ends inside a lane is stored by that lane; a
        // lane's first row may continue the previous lane's last one, and the run of lanes that
        // have nothing but that row is summed with a segmented scan - the row is then stored
        // once, by the lane where it ends.  No two lanes store the same row, and the tile
        // receives this chunk only, so plain stores do.
        auto entries_private = [&](auto load_x, auto split) {
            static_assert(kSparseChunksPerWave == 1, "a wavefront's tile takes one chunk: plain stores");
            constexpr uint32_t kNone = 0xffffffffu;
            float *tile = ytile + (size_t)wave * L.bh * BT;
            // the lane's first row is that of its first entry (kNone for a lane without a record)
            uint32_t first_row = kNone;
            if (y.n > 0) {
                uint32_t unused;
                split(st.sum + (y.z[0] & 0xffu), first_row, unused);
            }
            uint32_t cur = first_row;
            bool several = false;                       // the lane has left its first row
            float acc[BT], head[BT];
#pragma unroll
            for (int b = 0; b < BT; ++b) acc[b] = head[b] = 0.0f;
            // A change of row: the sum so far is stored, except the first one, which is kept - the
            // first row may have begun in the lanes before.  For one and two images that
            // distinction costs more than it saves: every sum is stored, the first row's too, and
            // that one is read back after the loop and written over with the sum over all its
            // lanes (one image: 33.9 -> 32.5 us per step of the
            // AlexNet-shaped stack; four images: 42.2 -> 43.2, so not there).
            auto enter_row = [&](uint32_t r) {
                if (r != cur) {
                    if (BT <= 2 || several) {
#pragma unroll
                        for (int b = 0; b < BT; ++b) tile[b * L.bh + cur] = acc[b];
                    }
#pragma unroll
                    for (int b = 0; b < BT; ++b) {
                        if (BT > 2) head[b] = several ? head[b] : acc[b];
                        acc[b] = 0.0f;
                    }
                    several = true;
                    cur = r;
                }
            };
            constexpr int G = BT <= 2 || BT > 8 ? 1 : 3;
            if constexpr (G == 1) {
                for_each_entry<false>(y, st.sum, [&](uint32_t, uint32_t v, uint32_t, uint32_t pos) {
                    uint32_t r, cc;
                    split(pos, r, cc);
                    enter_row(r);
                    const float w = s.T.cb[v];
                    float x[BT];
                    load_x((int)cc, x);
#pragma unroll
                    for (int b = 0; b < BT; ++b) acc[b] += w * x[b];
                });
            } else {
                // the codebook and activation reads of G entries go out together: the row logic
                // is all branches, behind which the compiler leaves each read where it is used
                uint32_t rows[G];
                float ws[G], xv[G][BT];
                for_each_entry_grouped<G>(y, st.sum, [&](int u, uint32_t v, uint32_t pos) {
                    uint32_t cc;
                    split(pos, rows[u], cc);
                    ws[u] = s.T.cb[v];
                    load_x((int)cc, xv[u]);
                }, [&](int u) {
                    enter_row(rows[u]);
#pragma unroll
                    for (int b = 0; b < BT; ++b) acc[b] += ws[u] * xv[u][b];
                });
            }
            // cur: the lane's last row (kNone for a lane without a record), acc its sum so far
            // (every lane takes part in the exchange: a lane that sat it out would hand its
            // neighbour a zero)
            const uint32_t from_prev = (uint32_t)__shfl_up((int)cur, 1), from_next = (uint32_t)__shfl_down((int)first_row, 1);
            const uint32_t prev_last = lane == 0 ? kNone : from_prev;
            const uint32_t next_first = lane == 63 ? kNone : from_next;
            const bool joins = first_row != kNone && first_row == prev_last;
            wave_segmented_sums<BT>(acc, !(joins && !several));
            float before[BT];                           // the run that ends in the lane before
#pragma unroll
            for (int b = 0; b < BT; ++b) before[b] = __shfl_up(acc[b], 1);
            if (several) {
#pragma unroll
                for (int b = 0; b < BT; ++b) {
                    if (BT <= 2) head[b] = tile[b * L.bh + first_row];       // (stored in the loop, by this lane)
                    tile[b * L.bh + first_row] = joins ? head[b] + before[b] : head[b];
                }
            }
            if (cur != kNone && next_first != cur) {
#pragma unroll
                for (int b = 0; b < BT; ++b) tile[b * L.bh + cur] = acc[b];
            }
        };
        auto entries = [&](auto load_x, auto split) {
            if (priv) entries_private(load_x, split);
            else entries_shared(load_x, split);
        };
        auto with_split = [&](auto load_x) {
            if (g.shift >= 0 && priv) {
                // (rows are used for a lane's own entries only here, and those lie inside the block:
                // checked when the layer was loaded)
                const uint32_t sh = (uint32_t)g.shift, cmask = (uint32_t)g.bwp - 1u;
                entries_private(load_x, [&](uint32_t pos, uint32_t &r, uint32_t &cc) { r = pos >> sh; cc = pos & cmask; });
            } else if (g.shift >= 0) {
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
                for (int q = 0; q < BT / kW; ++q) load_floats<kW>(xs + (xoff + cc) * BT + x_group<BT>(xoff + cc, q) * kW, x + q * kW);
            });
        } else {
            const float *xg = X + g.col_id;
            with_split([&](int cc, float (&x)[BT]) {
#pragma unroll
                for (int b = 0; b < BT; ++b) x[b] = b < nb ? xg[(size_t)b * L.K + cc] : 0.0f;
            });
        }
    }
    __syncthreads();
    float *mine = part + (size_t)wg * L.bh * BT;
    // (tiles added in wavefront order: the same every run; four outputs per thread where a tile's size allows)
    const int per_tile = L.bh * BT;
    if (BT >= 4) {
        for (int t = threadIdx.x; t < per_tile / 4; t += blockDim.x) {
            float4 v[kWaves];
#pragma unroll
            for (int w = 0; w < kWaves; ++w) v[w] = w < n_tiles ? ((const float4 *)(ytile + (size_t)w * per_tile))[t] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            float4 sum = v[0];
#pragma unroll
            for (int w = 1; w < kWaves; ++w)
                if (w < n_tiles) { sum.x += v[w].x; sum.y += v[w].y; sum.z += v[w].z; sum.w += v[w].w; }
            ((float4 *)mine)[t] = sum;
        }
    } else {
        for (int t = threadIdx.x; t < per_tile; t += blockDim.x) {
            float sum = ytile[t];
            for (int w = 1; w < n_tiles; ++w) sum += ytile[(size_t)w * per_tile + t];
            mine[t] = sum;
        }
    }
}

template <int BT, bool FOLD>
__global__ __launch_bounds__(kThreads) void fc_sparse_kernel(LayerDev L, const float *__restrict__ X, float *part,
                                                             int wg_per_panel, int xcap, PrevSlots prev, int nb)
{
    fc_sparse_body<BT, FOLD>(L, X, part, wg_per_panel, xcap, prev, blockIdx.x, nb);
}

// Several layers of one shape in one grid (the same layer of several models, or layers
// whose inputs do not depend on each other): workgroups wgs_per_layer i ..
// wgs_per_layer (i + 1) - 1 do layer i's share of Algorithm 2, from its own input
// (x_stride floats apart; 0: one input for all) into its own partial tiles.
template <int BT>
__global__ __launch_bounds__(kThreads) void fc_sparse_group_kernel(const LayerDev *__restrict__ table, uint32_t wgs_per_layer,
                                                                   const float *__restrict__ X, size_t x_stride, float *part,
                                                                   size_t part_stride, int wg_per_panel, int xcap)
{
    const uint32_t job = blockIdx.x / wgs_per_layer, wg = blockIdx.x - job * wgs_per_layer;
    const LayerDev L = table[job];
    fc_sparse_body<BT, false>(L, X + job * x_stride, part + job * part_stride, wg_per_panel, xcap,
                       PrevSlots{nullptr, nullptr, nullptr, 1, 0, 0, 0}, wg, BT);
}

// Finishes the sparse path: adds up the partial tiles of each block row in a fixed
// order, then bias and activation (Eq. 1): Y[b][row] = act(sum_j part[p][j][b][r] + v[row]).
// One workgroup per (block row, image).  The kernel is a chain of memory latencies and
// nothing else, so it is laid out to have few links: the threads form as many groups
// (slices) as fit next to one pass over the rows, slice s adds slots s, s + slices, ...
// with twelve loads in flight, LDS adds the slices in order.
constexpr int kRedThreads = 512;

__device__ __forceinline__ void fc_reduce_body(const LayerDev &L, const float *__restrict__ part, const float *__restrict__ bias,
                                               float *Y, int B, int part_b, int wg_per_panel, int relu, int wg)
{
    __shared__ float slice_sum[kRedThreads];
    const int p = wg / B, b = wg - p * B;
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

__global__ __launch_bounds__(kRedThreads) void fc_reduce_kernel(LayerDev L, const float *__restrict__ part,
                                                                const float *__restrict__ bias, float *Y, int B,
                                                                int part_b, int wg_per_panel, int relu)
{
    fc_reduce_body(L, part, bias, Y, B, part_b, wg_per_panel, relu, (int)blockIdx.x);
}

// The finishing kernel for fc_sparse_group_kernel: layer i's outputs at Y + i * y_stride,
// its bias (if any) at bias + i * bias_stride.
__global__ __launch_bounds__(kRedThreads) void fc_reduce_group_kernel(const LayerDev *__restrict__ table, int wgs_per_layer,
                                                                      const float *__restrict__ part, size_t part_stride,
                                                                      const float *__restrict__ bias, size_t bias_stride, float *Y,
                                                                      size_t y_stride, int B, int wg_per_panel, int relu)
{
    const int job = (int)blockIdx.x / wgs_per_layer, wg = (int)blockIdx.x - job * wgs_per_layer;
    const LayerDev L = table[job];
    fc_reduce_body(L, part + job * part_stride, bias ? bias + job * bias_stride : nullptr, Y + job * y_stride, B, B, wg_per_panel, relu,
                   wg);
}
