// Convolution as a matrix product without the column matrix in memory (Sec. III-A builds
// it; here the receptive fields are gathered straight into LDS): conv_mfma_kernel.
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

// Workgroup = (block row p of the filters, split j of its blocks, tile of 128 columns =
// image x output pixel) of wavefronts in two roles that meet at one barrier per block,
// as in fc_mfma_kernel, with the roles' data sources exchanged:
//   Gatherers (wavefronts 4-11) build, one block ahead, the 128 x 128 piece of the
//   column matrix that block i + 1 multiplies - row kk is (c, r, s) of the block's
//   column kk, column n an output pixel - in one of two LDS tiles, reading the NCHW
//   input directly (zero outside the image, past the last column and for rows the block
//   does not have).  A row is uniform per wavefront, a lane owns two columns (l and l + 64:
//   the 64 lanes of a load read neighbouring pixels) for the workgroup's whole life, so
//   where its pixels sit in the input, and which filter taps
//   fall outside the image there, is worked out once (COMBINED: one bit per tap, for
//   filters of at most 32 taps; else one bit per filter row and one per filter column).
//   What a row is - its offset from a receptive field's corner, its tap - comes from the
//   table that decode_tiles_kernel writes (`rows`), read with uniform loads.
//   Multipliers (wavefronts 0-3, one per SIMD): wavefront w owns filter rows 32w..32w+31
//   and all 128 columns in four 32 x 32 accumulators (other divisions for lower blocks,
//   below), with the operand layout of fc_mfma_kernel<4> - but the weights come from device memory (every block decoded
//   once per call by decode_tiles_kernel, in fragment order: a lane's four steps of one
//   row are one 16-byte load, 32 lanes contiguous) and the activations from LDS.
constexpr int kConvGatherers = 8;
constexpr int kConvThreads = (4 + kConvGatherers) * 64;
constexpr int kConvColumns = kTile;                        // columns per workgroup
constexpr int kActStride = kTile + 4;                      // floats per row of an activation tile (16-byte rows, skewed)
constexpr int kActTileFloats = kTile * kActStride;
constexpr int kConvLdsBytes = 2 * kActTileFloats * 4;
constexpr int kConvWAhead = 8;                             // 16-byte weight loads in flight per lane (four steps each)
constexpr int kConvAAhead = 4;                             // steps of activations read ahead from LDS

template <bool COMBINED, int S, int Q>
__global__ __launch_bounds__(kConvThreads) void conv_mfma_kernel(LayerDev L, const float *__restrict__ X, const float *__restrict__ wt,
                                                                 const uint2 *__restrict__ rows, float *part, ConvGeom cg, int n_cols,
                                                                 int Np, int splits, int panels_per_group, DirectOut out)
{
    extern __shared__ __attribute__((aligned(16))) float act[];        // [2][kTile][kActStride]
    const int nbt = Np / kConvColumns;
    const int nb = (int)blockIdx.x % nbt;
    const int pj = (int)blockIdx.x / nbt;
    const int p = pj / splits, j = pj % splits;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const int blk_lo = (int)(((int64_t)L.nbw * j) / splits), blk_hi = (int)(((int64_t)L.nbw * (j + 1)) / splits);
    const uint32_t pb0 = (uint32_t)p * (uint32_t)L.nbw;

    if (wave >= 4) {
        const int d = wave - 4;
        const int pq = cg.P * cg.Q, plane = cg.H * cg.W;
        const int c0 = (p / panels_per_group) * cg.Cg;              // the filter group's input channels
        // The input is read through a buffer descriptor that starts at the tile's first
        // image, channel c0, moved back by the padding so that a receptive field's corner
        // has a non-negative offset (the launcher keeps 129 images under 2^29 elements, so
        // byte offsets stay below 2^31), and ends with the input: a load past its end returns
        // zero.  That is also how an element outside the image is read - its offset is turned
        // into 0xffffffff - so a gathered element costs a bit test, an add, an or and a load,
        // with no branch.  (Word 3 of the descriptor: 32-bit elements, plain addressing.)
        const int img0 = nb * kConvColumns / pq;
        const int n_img = (n_cols + pq - 1) / pq;
        const int64_t back = (int64_t)cg.pad * cg.W + cg.pad;
        const int64_t span = (((int64_t)(n_img - img0) * cg.C - c0) * plane + back) * (int64_t)sizeof(float);
        const __amdgpu_buffer_rsrc_t xb = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(X + ((int64_t)img0 * cg.C + c0) * plane - back), 0, (int)std::min<int64_t>(span, 0x7fffffff), 0x00020000);
        // The lane's two columns: byte offset of the corner of each pixel's receptive field,
        // and which (r, s) fall outside the image - one bit per (r, s) when the filter has
        // at most 32 taps, else one per r and one per s.  Columns past the last are all outside.
        uint32_t at[2], bad[2], bad_s[2];
        {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int n = nb * kConvColumns + lane + 64 * i;
                const int img = n / pq;
                const int o = n - img * pq;
                const int oy = o / cg.Q, ox = o - oy * cg.Q;
                const int y0 = oy * cg.stride - cg.pad, x0 = ox * cg.stride - cg.pad;
                at[i] = (uint32_t)((img - img0) * cg.C * plane + oy * cg.stride * cg.W + ox * cg.stride) * (uint32_t)sizeof(float);
                uint32_t rb = 0, sb = 0;
                for (int r = 0; r < cg.R; ++r) rb |= (uint32_t)((unsigned)(y0 + r) >= (unsigned)cg.H) << r;
                for (int sx = 0; sx < cg.S; ++sx) sb |= (uint32_t)((unsigned)(x0 + sx) >= (unsigned)cg.W) << sx;
                if (n >= n_cols) rb = sb = 0xffffffffu;
                if (COMBINED) {
                    const uint32_t all_s = cg.S >= 32 ? 0xffffffffu : (1u << cg.S) - 1u;
                    uint32_t both = 0;
                    for (int r = 0; r < cg.R; ++r) both |= ((rb >> r) & 1u ? all_s : (sb & all_s)) << (r * cg.S);
                    rb = both;
                }
                bad[i] = rb;
                bad_s[i] = sb;
            }
        }
        // Wavefront d gathers rows 16 d .. 16 d + 15 of a piece; what a row is comes from
        // the table (uniform loads), so a row costs no arithmetic of its own.
        constexpr int kRows = kTile / kConvGatherers;
        auto fill = [&](int bi, float *tile) {
            const uint2 *rp = rows + (bi * kTile + kRows * d);
            float v[kRows][2];
#pragma unroll
            for (int jj = 0; jj < kRows; ++jj) {
                const uint2 e = rp[jj];
                const uint32_t no_row = (uint32_t)((int)e.y >> 31);
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const uint32_t out = COMBINED ? (uint32_t)__builtin_amdgcn_sbfe(bad[i], e.y & 0xffu, 1)
                                                  : (uint32_t)(__builtin_amdgcn_sbfe(bad[i], e.y & 0xffu, 1) |
                                                               __builtin_amdgcn_sbfe(bad_s[i], (e.y >> 8) & 0xffu, 1));
                    v[jj][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(xb, (int)((at[i] + e.x) | out | no_row), 0, 0));
                }
            }
#pragma unroll
            for (int jj = 0; jj < kRows; ++jj) {
                tile[(kRows * d + jj) * kActStride + lane] = v[jj][0];
                tile[(kRows * d + jj) * kActStride + lane + 64] = v[jj][1];
            }
        };
        if (blk_lo < blk_hi) fill(blk_lo, act);
        __syncthreads();
        for (int bi = blk_lo; bi < blk_hi; ++bi) {
            if (bi + 1 < blk_hi) fill(bi + 1, act + (((bi - blk_lo) & 1) ^ 1) * kActTileFloats);
            __syncthreads();
        }
        return;
    }

    // S x Q accumulators of 32 filter rows x 32 columns per multiplying wavefront w, by the
    // height of the layer's blocks:
    //   up to 128 rows (S = 1, Q = 4): rows 32 w .. 32 w + 31, all 128 columns;
    //   up to  96 rows (S = 3, Q = 1): all 96 rows, columns 32 w .. 32 w + 31;
    //   up to  64 rows (S = 1, Q = 2): rows 32 (w % 2) .., columns 64 (w / 2) .. + 63;
    // so that no wavefront multiplies rows that no block has.  Accumulator (s, q) holds,
    // for element e of lane (kl, m), filter row 32 (sbase + s) + m and column
    // cbase + Q i + q of the tile, i = 8 (e / 4) + 4 kl + e % 4.
    const int sbase = S == 3 ? 0 : (Q == 4 ? wave : wave & 1);
    const int cbase = S == 3 ? 32 * wave : (Q == 4 ? 0 : 64 * (wave >> 1));
    constexpr int kWA = S == 3 ? kConvWAhead / 2 : kConvWAhead;     // weight loads in flight per strip
    floatx16 acc[S][Q];
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int q = 0; q < Q; ++q) acc[s][q] = floatx16{0};
    const int kl = lane >> 5, m = lane & 31;
    // piece (column group 16 kl + g, row 32 strip + m) of a tile in fragment order: steps
    // 4 g .. 4 g + 3 of this lane's row; groups follow each other 128 pieces apart, strips 32
    const float4 *wf = (const float4 *)wt + ((size_t)(pb0 + (uint32_t)blk_lo) * (kTile / 4) + 16 * kl) * kTile + 32 * sbase + m;
    float4 w[S][kWA];
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int i = 0; i < kWA; ++i) w[s][i] = wf[i * kTile + 32 * s];
    __syncthreads();                                        // first piece of the column matrix gathered
    for (int bi = blk_lo; bi < blk_hi; ++bi) {
        const float *ap = act + ((bi - blk_lo) & 1) * kActTileFloats + 64 * kl * kActStride + cbase + Q * m;
        // the pieces loaded towards the end of this block are the next block's first ones
        // (the last block re-reads its own: valid memory, never multiplied)
        const float4 *wnext = bi + 1 < blk_hi ? wf + (kTile / 4) * kTile : wf;
        float a[kConvAAhead][Q];
#pragma unroll
        for (int i = 0; i < kConvAAhead; ++i) load_floats<Q>(ap + i * kActStride, a[i]);
#pragma unroll
        for (int g = 0; g < kTile / 8; ++g) {
            // program order is pinned (scheduling barriers): left alone, the compiler sinks the
            // loads to just before their use and their latency lands in front of the multiplies
            float4 wv[S];
#pragma unroll
            for (int s = 0; s < S; ++s) wv[s] = w[s][g % kWA];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < S; ++s)
                w[s][g % kWA] = g + kWA < kTile / 8 ? wf[(g + kWA) * kTile + 32 * s] : wnext[(g + kWA - kTile / 8) * kTile + 32 * s];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int st = 4 * g + u;
                float av[Q];
#pragma unroll
                for (int q = 0; q < Q; ++q) av[q] = a[st % kConvAAhead][q];
                __builtin_amdgcn_sched_barrier(0);
                if (st + kConvAAhead < kTile / 2) load_floats<Q>(ap + (st + kConvAAhead) * kActStride, a[st % kConvAAhead]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    const float wu = u == 0 ? wv[s].x : u == 1 ? wv[s].y : u == 2 ? wv[s].z : wv[s].w;
#pragma unroll
                    for (int q = 0; q < Q; ++q) acc[s][q] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q], wu, acc[s][q], 0, 0, 0);
                }
            }
        }
        wf = wnext;
        __syncthreads();                                    // done with this piece
    }

    const int row_id = p * L.bh;
    const int block_rows = min(L.bh, L.M - row_id);
    if (!out.Y) {
        // the workgroup's partial tile for the finishing kernel: 32 lanes write 32 consecutive rows of a column
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (32 * (sbase + s) + m >= block_rows) continue;
            float *mine = part + ((size_t)pj * Np + (size_t)nb * kConvColumns + cbase) * L.bh + 32 * (sbase + s) + m;
#pragma unroll
            for (int e = 0; e < 16; ++e)
#pragma unroll
                for (int q = 0; q < Q; ++q) mine[(size_t)(Q * (8 * (e / 4) + 4 * kl + (e & 3)) + q) * L.bh] = acc[s][q][e];
        }
        return;
    }
    // The finished output (block rows that are not split).  The output runs along the
    // columns, the accumulators along the rows: the wavefront turns its 32 S x 32 Q piece in
    // its own part of LDS (the tiles are free: the last barrier was every wavefront's last
    // use of them), then writes each filter row's columns as one run - two rows at a time
    // where a row has 32 columns - bias (lane l holds that of row l % 32 of each strip) and
    // activation on the way.
    constexpr int kCols = 32 * Q, kStride = kCols + 1;
    constexpr int kPerLane = kCols > 64 ? kCols / 64 : 1;       // columns of a row per lane
    constexpr int kRowsAtOnce = kCols < 64 ? 64 / kCols : 1;    // rows per pass of the wavefront
    float *t = act + wave * (32 * S) * kStride;
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int e = 0; e < 16; ++e)
#pragma unroll
            for (int q = 0; q < Q; ++q) t[(32 * s + m) * kStride + Q * (8 * (e / 4) + 4 * kl + (e & 3)) + q] = acc[s][q][e];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const int my_col = kRowsAtOnce > 1 ? lane % kCols : lane, my_row = kRowsAtOnce > 1 ? lane / kCols : 0;
    size_t y_at[kPerLane];
    bool live[kPerLane];
#pragma unroll
    for (int i = 0; i < kPerLane; ++i) {
        const int c = nb * kConvColumns + cbase + my_col + 64 * i;
        live[i] = c < out.ncols;
        y_at[i] = ((size_t)(c / out.pq) * L.M + row_id) * out.pq + (c % out.pq);
    }
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const int first = 32 * (sbase + s);                       // the strip's first row in the block
        const int n_rows = min(32, block_rows - first);
        const float bias_l = out.bias && m < n_rows ? out.bias[row_id + first + m] : 0.0f;
        for (int r0 = 0; r0 < n_rows; r0 += 8 * kRowsAtOnce) {
            float y[8][kPerLane];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int ru = min(r0 + kRowsAtOnce * u, 31);     // uniform; this lane's row is ru + my_row
                const float b0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bias_l), ru));
                const float b1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bias_l), min(ru + 1, 31)));
                const int rr = min(ru + my_row, 31);
#pragma unroll
                for (int i = 0; i < kPerLane; ++i) y[u][i] = t[(32 * s + rr) * kStride + my_col + 64 * i] + (my_row ? b1 : b0);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int rr = r0 + kRowsAtOnce * u + my_row;
                if (rr >= n_rows) continue;
#pragma unroll
                for (int i = 0; i < kPerLane; ++i)
                    if (live[i]) out.Y[y_at[i] + (size_t)(first + rr) * out.pq] = out.relu ? fmaxf(y[u][i], 0.0f) : y[u][i];
            }
        }
    }
}
