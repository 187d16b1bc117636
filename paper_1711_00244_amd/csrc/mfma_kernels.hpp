// Dense-tile path on the fp32 matrix cores: activation layouts, the decoder role shared by the dense-tile kernels, fc_mfma_kernel.
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

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

constexpr int kIm2colRows = 16;          // most rows of XT a workgroup of im2col_pad_kernel writes for its columns (a power of two)

__global__ __launch_bounds__(256) void im2col_pad_kernel(const float *__restrict__ X, float *XT, ConvGeom cg, size_t x_stride,
                                                         int n_cols, int Np, int bw, int K, int grp0, int rows_per_wg)
{
    const int c0 = (grp0 + (int)blockIdx.z) * cg.Cg;        // filter group grp0 + blockIdx.z: its input channels, matrix blockIdx.z
    XT += (size_t)blockIdx.z * x_stride;
    const int pq = cg.P * cg.Q;
    const int plane = cg.H * cg.W;
    const int row0 = (int)blockIdx.y * rows_per_wg;
    // A thread writes four consecutive columns (Np is a multiple of the 32-column
    // accumulator) of rows_per_wg rows: where its four output pixels sit in the input
    // is worked out once, a row (c, r, s) then only shifts that by a uniform offset.
    for (int n4 = blockIdx.x * blockDim.x + threadIdx.x; n4 < Np / 4; n4 += gridDim.x * blockDim.x) {
        const int n = 4 * n4;
        int y0[4], x0[4];
        size_t at[4];                                       // offset of (y0, x0) of the pixel's image, channel 0
        {
            int img = n / pq;
            const int o = n - img * pq;
            int oy = o / cg.Q, ox = o - oy * cg.Q;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // columns past the last one get coordinates that no (r, s) brings inside the image
                y0[i] = n + i < n_cols ? oy * cg.stride - cg.pad : -(1 << 20);
                x0[i] = ox * cg.stride - cg.pad;
                at[i] = (size_t)img * cg.C * plane + (size_t)((int64_t)y0[i] * cg.W + x0[i]);
                if (++ox == cg.Q) {
                    ox = 0;
                    if (++oy == cg.P) { oy = 0; ++img; }
                }
            }
        }
        for (int rr = 0; rr < rows_per_wg; ++rr) {
            const int k = xt_row_to_k(row0 + rr, bw, K);    // (c, r, s) of this row, or a padding row: uniform
            float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (k >= 0) {
                const int s = k % cg.S, r = (k / cg.S) % cg.R, c = k / (cg.S * cg.R);
                const size_t shift = (size_t)(c0 + c) * plane + (size_t)(r * cg.W + s);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if ((unsigned)(y0[i] + r) < (unsigned)cg.H && (unsigned)(x0[i] + s) < (unsigned)cg.W) v[i] = X[at[i] + shift];
            }
            ((float4 *)(XT + (size_t)(row0 + rr) * Np))[n4] = make_float4(v[0], v[1], v[2], v[3]);
        }
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
// block.  The two buffers are BUF_FLOATS floats apart; look(v) reads what stands for
// value index v (the codebook entry, or its two bf16 halves) and put(buffer, row,
// column, that) places it (in the tile, or in two half tiles).  With CLEAR_BARRIER the multipliers clear a used tile between two barriers
// (their rows are shared), else right after their last read of their own rows.
// Called by wavefronts 4 .. 4 + DEC - 1.
template <int DEC, bool CLEAR_BARRIER, int BUF_FLOATS, class Look, class Put>
__device__ __forceinline__ void decoder_role(const LayerDev &L, const Smem &s, float *tiles, int blk_lo, int blk_hi, uint32_t pb0,
                                             int wave, int lane, Look look, Put put)
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
                place_entries(y, st.sum, look,
                              [&](uint32_t pos, auto w) { put(tile, min(pos >> sh, rmax), pos & cmask, w); });
            } else {
                for_each_entry(y, st.sum, [&](uint32_t, uint32_t v, uint32_t, uint32_t pos) {
                    uint32_t r, cc;
                    split_pos(pos, g, r, cc);
                    if (v != 0 && cc < (uint32_t)kTile) put(tile, r, cc, look(v));
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

// Every block of the layer decoded once into a dense 128 x 128 fp32 tile in device
// memory (Algorithm 2 steps 5-9 for all blocks; rows and columns a block does not have
// are zero).  One workgroup per block, a chunk per wavefront at a time, the tile built
// in LDS and written out in one piece as tiles_out[block][column / 4][row][column % 4]:
// the order in which the lanes of a multiplying wavefront of conv_mfma_kernel take their
// 16-byte pieces of a tile straight from device memory.  For a convolution, where
// hundreds of column tiles multiply the same few blocks.
//
// The launch also writes what the gatherers of conv_mfma_kernel need to know of a row
// of the column matrix, for every row of every 128 x 128 piece (piece bi, row kk = column
// bi bw + kk of the layer = (c, r, s)): x = byte offset of (c, r, s) from a receptive
// field's corner at channel 0, y = which bit of a column's tap masks says whether the tap
// is outside the image (r S + s when `combined`, else r | s << 8), with the top bit set
// for a row the piece does not have.  n_rows entries, one per thread of the launch's
// first workgroups (a layer has at least as many blocks as pieces).
// Sixteen wavefronts: a dense block has up to 35 chunks, and the launch is as long as its rounds of chunks.
constexpr int kTileDecodeWaves = 16;
constexpr int kTileDecodeThreads = kTileDecodeWaves * 64;

__global__ __launch_bounds__(kTileDecodeThreads) void decode_tiles_kernel(LayerDev L, float *tiles_out, ConvGeom cg, int n_rows, int combined,
                                                                uint2 *rows)
{
    {
        const int t = (int)(blockIdx.x * kTileDecodeThreads + threadIdx.x);
        if (t < n_rows) {
            const int kk = t % kTile, k = (t / kTile) * L.bw + kk;
            uint2 e = make_uint2(0u, 0x80000000u);
            if (kk < L.bw && k < L.K) {
                const int s = k % cg.S, r = (k / cg.S) % cg.R, c = k / (cg.S * cg.R);
                e.x = (uint32_t)(c * cg.H * cg.W + r * cg.W + s) * (uint32_t)sizeof(float);
                e.y = combined ? (uint32_t)(r * cg.S + s) : (uint32_t)(r | s << 8);
            }
            rows[t] = e;
        }
    }
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    float *tile = s.extra;                                  // [kTile][kWStride]
    const uint32_t b = blockIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const uint32_t c0 = L.block_chunk[b], c1 = L.block_chunk[b + 1];
    TableRegs tr;
    if (threadIdx.x < kThreads) tr = fetch_tables(L);           // the table image is copied by kThreads threads
    for (int t = threadIdx.x; t < kTile * kWStride / 4; t += kTileDecodeThreads) ((uint4 *)tile)[t] = uint4{0, 0, 0, 0};
    if (threadIdx.x < kThreads) store_tables(s, L, tr);
    __syncthreads();
    const BlockGeom g = block_geom(L, b);
    for (uint32_t c = c0 + (uint32_t)wave; c < c1; c += kTileDecodeWaves) {       // uniform per wavefront
        const ChunkHead h = load_head(L, c);
        const Symbols y = decode_record(load_record(L, h, lane), s.T);
        const LaneStart st = lane_starts(y, h.m.pos0);
        for_each_entry(y, st.sum, [&](uint32_t, uint32_t v, uint32_t, uint32_t pos) {
            uint32_t r, cc;
            split_pos(pos, g, r, cc);
            if (v != 0 && cc < (uint32_t)kTile) tile[r * kWStride + cc] = s.T.cb[v];
        });
    }
    __syncthreads();
    uint4 *dst = (uint4 *)(tiles_out + (size_t)b * kTile * kTile);
    const uint4 *src = (const uint4 *)tile;
    for (int t = threadIdx.x; t < kTile * kTile / 4; t += kTileDecodeThreads) {
        // piece t of the output: row t % 128, columns 4 (t / 128) .. 4 (t / 128) + 3
        dst[t] = src[(t % kTile) * (kWStride / 4) + t / kTile];
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

// Where a convolution's block rows are not split, nothing is left to add up and the
// kernel finishes the output itself (bias, activation, NCHW) instead of writing
// partial tiles for the finishing kernel: Y is null otherwise.
struct DirectOut {
    float *Y;              // batch x M x pq, or null
    const float *bias;     // M values or null
    int ncols, pq, relu;   // real columns (image x pixel), pixels per image
};

// What a multiplying wavefront does with its finished accumulators: accumulator 4 v + q,
// element e of lane l holds column 128 v + kVecW (8 (e / 4) + 4 (l / 32) + e % 4) + q of the
// workgroup's tile for weight row 32 wave + l % 32.  Either the finished output (out.Y:
// bias, activation, NCHW, through `lds`, which must be free: every wavefront has passed
// its last barrier) or the workgroup's partial tile for the finishing kernel.
template <int NQ>
__device__ __forceinline__ void store_accumulators(const floatx16 (&acc)[NQ], const LayerDev &L, float *lds, float *part,
                                                   const DirectOut &out, int pj, int p, int nb, int Bp, int wave, int lane)
{
    constexpr int kImages = MfmaShape<NQ>::kImages;
    constexpr int kVecW = MfmaShape<NQ>::kVecW, kVecs = MfmaShape<NQ>::kVecs;
    const int kl = lane >> 5, m = lane & 31;
    float *tiles = lds;
    const int r = wave * 32 + m;
    if (out.Y) {
        // The output runs along the columns, the accumulators along the rows: turn the
        // wavefront's 32 x kImages piece in LDS (the weight tiles are free now; the last
        // barrier above was every wavefront's last use of them), then write each row's
        // columns in runs, bias and activation on the way.
        constexpr int kStride = kImages + 1;
        float *t = tiles + wave * 32 * kStride;
#pragma unroll
        for (int v = 0; v < kVecs; ++v) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int slot = 8 * (e / 4) + 4 * kl + (e & 3);
#pragma unroll
                for (int q = 0; q < kVecW; ++q) t[m * kStride + kTile * v + kVecW * slot + q] = acc[4 * v + q][e];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const int row_id = p * L.bh;
        const int rows = min(32, min(L.bh, L.M - row_id) - wave * 32);
        // a lane's columns are the same for every row: where they sit in Y is worked out once
        constexpr int kMine = (kImages + 63) / 64;
        size_t at[kMine];
        bool live[kMine];
#pragma unroll
        for (int i = 0; i < kMine; ++i) {
            const int c = nb * kImages + lane + 64 * i;
            live[i] = lane + 64 * i < kImages && c < out.ncols;
            at[i] = ((size_t)(c / out.pq) * L.M + row_id + wave * 32) * out.pq + (c % out.pq);
        }
        // lane l holds the bias of the wavefront's row l % 32; eight rows at a time, their
        // LDS reads ahead of their stores
        const float bias_l = out.bias && m < rows ? out.bias[row_id + wave * 32 + m] : 0.0f;
        for (int r0 = 0; r0 < rows; r0 += 8) {
            float y[8][kMine];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int rr = min(r0 + u, rows - 1);
                const float bv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bias_l), rr));
#pragma unroll
                for (int i = 0; i < kMine; ++i) y[u][i] = t[rr * kStride + lane + 64 * i] + bv;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (r0 + u >= rows) break;
#pragma unroll
                for (int i = 0; i < kMine; ++i)
                    if (live[i]) out.Y[at[i] + (size_t)(r0 + u) * out.pq] = out.relu ? fmaxf(y[u][i], 0.0f) : y[u][i];
            }
        }
        return;
    }
    // 32 lanes write 32 consecutive floats of the workgroup's partial tile
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

template <int NQ>
__global__ __launch_bounds__(MfmaShape<NQ>::kThreads) void fc_mfma_kernel(LayerDev L, const float *__restrict__ XT, float *part,
                                                                         int splits, int Bp, int panels_per_x, size_t x_stride,
                                                                         DirectOut out)
{
    constexpr int kMfmaDecoders = MfmaShape<NQ>::kDecoders;
    constexpr int kMfmaThreads = MfmaShape<NQ>::kThreads;
    constexpr int kAhead = MfmaShape<NQ>::kAhead;
    constexpr int kImages = MfmaShape<NQ>::kImages;
    constexpr int kVecW = MfmaShape<NQ>::kVecW, kVecs = MfmaShape<NQ>::kVecs;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    float *tiles = (float *)s.extra;                                  // [2][kTile rows][kWStride]
    const int nbt = Bp / kImages;
    const int nb = (int)blockIdx.x % nbt;
    const int pj = (int)blockIdx.x / nbt;
    const int p = L.panel0 + pj / splits, j = pj % splits;    // part slots are numbered from the launch's first block row
    // every panels_per_x block rows have an activation matrix of their own, x_stride
    // elements after the one before (the filter groups of a convolution)
    XT += (size_t)((pj / splits) / panels_per_x) * x_stride;
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
                                                             [&](uint32_t v) { return s.T.cb[v]; },
                                                             [&](float *tile, uint32_t r, uint32_t cc, float w) { tile[__umul24(r, (uint32_t)kWStride) + cc] = w; });
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
        float4 *wp = (float4 *)(cur + (wave * 32 + m) * kWStride + 64 * kl);
        float4 b_cur = wp[0];
        for (int ks = 0; ks < kTile / 2; ks += kAhead) {
            // steps are kept in program order (scheduling barriers): hoisting a group's
            // LDS reads or sinking its loads would put their latency in front of the
            // multiplies
#pragma unroll
            for (int h4 = 0; h4 < kAhead / 4; ++h4) {
                const float4 b_next = wp[min(ks / 4 + h4 + 1, kTile / 8 - 1)];
                // The four weights in b_cur are this lane's alone and have been read: zero them
                // now, behind the multiplies, so that the decoders get a clean tile back.
                wp[ks / 4 + h4] = float4{0.0f, 0.0f, 0.0f, 0.0f};
                __builtin_amdgcn_sched_barrier(0);          // the LDS accesses go out before these multiplies
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
        __syncthreads();                                    // done with this tile, and it is clean
    }
    store_accumulators<NQ>(acc, L, tiles, part, out, pj, p, nb, Bp, wave, lane);
}
