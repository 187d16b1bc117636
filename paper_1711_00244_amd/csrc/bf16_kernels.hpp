// Dense-tile path on the bf16 matrix cores (three products per fp32 product).
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

// ------------------------------------------------------------------------- //
// dense tiles on the bf16 matrix cores, three products per fp32 product
// ------------------------------------------------------------------------- //
// A weight w and an activation x are each split into two bf16 terms, w = wh + wl,
// x = xh + xl (round to nearest even; the residual of each is below 2^-16 of the value),
// and w x is taken as xh wh + xh wl + xl wh with fp32 accumulation in
// v_mfma_f32_32x32x16_bf16: three multiplies at sixteen times the fp32 rate.  What is
// dropped (xl wl and the two residuals) is below 3 * 2^-16 of |w x|.
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
                                                           int n_cols, int Np, int bw, int K, size_t plane_elems, int grp0)
{
    const int c0 = (grp0 + (int)blockIdx.z) * cg.Cg;
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
    const int p = L.panel0 + pj / splits, j = pj % splits;
    XB += (size_t)((pj / splits) / panels_per_x) * x_stride;            // one pair of planes per filter group
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    store_tables(s, L, fetch_tables(L));
    for (int t = threadIdx.x; t < 2 * kBf16BufFloats / 4; t += kNThreads) ((uint4 *)tiles)[t] = uint4{0, 0, 0, 0};
    for (int t = threadIdx.x; t < L.ncode; t += kNThreads) cbp[t] = bf16_split(L.codebook[t]);
    const int blk_lo = (int)(((int64_t)L.nbw * j) / splits), blk_hi = (int)(((int64_t)L.nbw * (j + 1)) / splits);
    const uint32_t pb0 = (uint32_t)p * (uint32_t)L.nbw;
    if (wave >= 4) {
        decoder_role<kDec, true, kBf16BufFloats>(L, s, tiles, blk_lo, blk_hi, pb0, wave, lane,
                                                 [&](uint32_t v) { return cbp[v]; },
                                                 [&](float *tile, uint32_t r, uint32_t cc, uint32_t w) {
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
