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
//   and all 128 columns in four 32 x 32 accumulators (HALF: 32 of 64 rows and 64 columns
//   in two), with the operand layout of fc_mfma_kernel<4> - but the weights come from device memory (every block decoded
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

template <bool COMBINED, bool HALF>
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

    // NA accumulators of 32 filter rows x 32 columns per multiplying wavefront.  Blocks of
    // up to 128 rows: wavefront w takes rows 32 w .. 32 w + 31 and all 128 columns (NA = 4,
    // accumulator q holds columns 4 i + q).  HALF, for layers whose blocks have at most 64
    // rows: wavefront w takes rows 32 (w % 2) .. and columns 64 (w / 2) .. + 63 (NA = 2,
    // accumulator q holds columns 64 (w / 2) + 2 i + q), so that no wavefront multiplies
    // rows that no block has.
    constexpr int NA = HALF ? 2 : 4;
    const int strip = HALF ? wave & 1 : wave, chalf = HALF ? wave >> 1 : 0;
    floatx16 acc[NA];
#pragma unroll
    for (int q = 0; q < NA; ++q) acc[q] = floatx16{0};
    const int kl = lane >> 5, m = lane & 31;
    // piece (column group 16 kl + g, row 32 strip + m) of a tile in fragment order: steps
    // 4 g .. 4 g + 3 of this lane's row; groups follow each other 128 pieces apart
    const float4 *wf = (const float4 *)wt + ((size_t)(pb0 + (uint32_t)blk_lo) * (kTile / 4) + 16 * kl) * kTile + 32 * strip + m;
    float4 w[kConvWAhead];
#pragma unroll
    for (int i = 0; i < kConvWAhead; ++i) w[i] = wf[i * kTile];
    __syncthreads();                                        // first piece of the column matrix gathered
    for (int bi = blk_lo; bi < blk_hi; ++bi) {
        const float *ap = act + ((bi - blk_lo) & 1) * kActTileFloats + 64 * kl * kActStride + 64 * chalf + NA * m;
        // the pieces loaded towards the end of this block are the next block's first ones
        // (the last block re-reads its own: valid memory, never multiplied)
        const float4 *wnext = bi + 1 < blk_hi ? wf + (kTile / 4) * kTile : wf;
        float a[kConvAAhead][NA];
#pragma unroll
        for (int i = 0; i < kConvAAhead; ++i) load_floats<NA>(ap + i * kActStride, a[i]);
#pragma unroll
        for (int g = 0; g < kTile / 8; ++g) {
            // program order is pinned (scheduling barriers): left alone, the compiler sinks the
            // loads to just before their use and their latency lands in front of the multiplies
            const float4 wv = w[g % kConvWAhead];
            __builtin_amdgcn_sched_barrier(0);
            w[g % kConvWAhead] = g + kConvWAhead < kTile / 8 ? wf[(g + kConvWAhead) * kTile] : wnext[(g + kConvWAhead - kTile / 8) * kTile];
            __builtin_amdgcn_sched_barrier(0);
            const float wu[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int s = 4 * g + u;
                float av[NA];
#pragma unroll
                for (int q = 0; q < NA; ++q) av[q] = a[s % kConvAAhead][q];
                __builtin_amdgcn_sched_barrier(0);
                if (s + kConvAAhead < kTile / 2) load_floats<NA>(ap + (s + kConvAAhead) * kActStride, a[s % kConvAAhead]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < NA; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[q], wu[u], acc[q], 0, 0, 0);
            }
        }
        wf = wnext;
        __syncthreads();                                    // done with this piece
    }
    if constexpr (!HALF) {
        store_accumulators<4>(acc, L, act, part, out, pj, p, nb, Np, wave, lane);
        return;
    } else {
    // HALF: accumulator q, element e of lane (kl, m) is column 64 chalf + 16 (e / 4) + 8 kl +
    // 2 (e % 4) + q of the tile for filter row 32 strip + m
    const int row_id = p * L.bh;
    const int n_rows = min(32, min(L.bh, L.M - row_id) - 32 * strip);
    if (!out.Y) {
        // the workgroup's partial tile: 32 lanes write 32 consecutive rows of a column
        if (m < n_rows) {
            float *mine = part + ((size_t)pj * Np + (size_t)nb * kConvColumns + 64 * chalf) * L.bh + 32 * strip + m;
#pragma unroll
            for (int e = 0; e < 16; ++e)
#pragma unroll
                for (int q = 0; q < NA; ++q) mine[(size_t)(16 * (e / 4) + 8 * kl + 2 * (e & 3) + q) * L.bh] = acc[q][e];
        }
        return;
    }
    // the finished output: the wavefront's 32 x 64 piece turned in its own part of LDS (the
    // tiles are free: the last barrier was every wavefront's last use of them), then each
    // filter row's 64 columns written as one run, bias (lane l holds that of row l % 32) and
    // activation on the way
    constexpr int kStride = 65;
    float *t = act + wave * 32 * kStride;
#pragma unroll
    for (int e = 0; e < 16; ++e)
#pragma unroll
        for (int q = 0; q < NA; ++q) t[m * kStride + 16 * (e / 4) + 8 * kl + 2 * (e & 3) + q] = acc[q][e];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    const int c = nb * kConvColumns + 64 * chalf + lane;        // this lane's column
    const bool live = c < out.ncols;
    const size_t y_at = ((size_t)(c / out.pq) * L.M + row_id + 32 * strip) * out.pq + (c % out.pq);
    const float bias_l = out.bias && m < n_rows ? out.bias[row_id + 32 * strip + m] : 0.0f;
    for (int r0 = 0; r0 < n_rows; r0 += 8) {
        float y[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int rr = min(r0 + u, n_rows - 1);
            y[u] = t[rr * kStride + lane] + __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bias_l), rr));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (r0 + u >= n_rows) break;
            if (live) out.Y[y_at + (size_t)(r0 + u) * out.pq] = out.relu ? fmaxf(y[u], 0.0f) : y[u];
        }
    }
    }
}
