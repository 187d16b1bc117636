// Large batches on the vector ALUs: the sparse product of Algorithm 2 step 12 as written -
// one multiply-add per surviving weight and image, no dense tile - with the images across
// the lanes.  fc_wide_kernel and its finishing kernel.
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

// Workgroup (block row p, split j of its blocks, image tile nb of 64 IPL images) of
// sixteen wavefronts in two roles that meet at one barrier per phase.
//   Decoders (wavefronts 12-15, one per SIMD) decode block i + 1 - a chunk per wavefront
//   at a time, decode / scan as everywhere - into an entry list in LDS: the block's
//   surviving weights in the order of the stream (row by row), 16 bits each (column in
//   the block, value index), the padding entries dropped; and a pointer array that says
//   where in the list each half row starts (half row h = 2 row + (column >= 64): the
//   positions of a block run row by row, so h never decreases along the list).
//   Multipliers (wavefronts 0-11) own kWideRows rows of the block row each and hold
//   their sums for all images of the tile in registers (lane l: images IPL l .. IPL l +
//   IPL - 1) for the whole split.  An entry is uniform across the wavefront: its column
//   picks a row of the activation slab in LDS ([column][image], one ds_read of IPL floats
//   per lane), its weight multiplies that into the sums of its row.  The rows are walked
//   in program order (so which registers a row's sums live in is static), a row's
//   entries in groups of four.
// The activations of a block's 128 columns and 256 images are 128 KB, so a block is
// taken in two phases of 64 columns (one for blocks of at most 64 columns): two slabs
// of 64 x (64 IPL) floats alternate, the slab of phase s + 1 is loaded during phase s
// by all sixteen wavefronts, and the half-row pointers give each phase its entries.
// The entry list and pointers of two blocks alternate likewise.
constexpr int kWideWaves = 16;
constexpr int kWideDecoders = 4;
constexpr int kWideMults = kWideWaves - kWideDecoders;
constexpr int kWideThreads = kWideWaves * 64;
constexpr int kWideRows = (kTile + kWideMults - 1) / kWideMults;       // rows of a block row per multiplying wavefront
constexpr int kHalf = 64;                                               // columns per slab
constexpr int kHalfKeys = 2 * kTile;                                    // half rows of a block
constexpr int kHalfPtrStride = (kHalfKeys + 1 + 7) / 8 * 8;             // 16-bit pointers per buffer, kept 16-byte aligned
constexpr int kSlabRowsPerWave = kHalf / kWideWaves;                    // rows of a slab each wavefront copies

// bytes of LDS after the table image: two pointer arrays, two entry lists, two slabs
static size_t wide_lds_bytes(size_t tables, int cap, int ipl)
{
    return tables + 2 * (size_t)kHalfPtrStride * 2 + 2 * (size_t)cap * 2 + 2 * (size_t)kHalf * 64 * ipl * 4;
}

// 1 in every byte of x that is not zero
__device__ __forceinline__ uint32_t nonzero_bytes(uint32_t x)
{
    return ((x | ((x & 0x7f7f7f7fu) + 0x7f7f7f7fu)) & 0x80808080u) >> 7;
}

// Half row of a position of block g: 2 row + (column >= kHalf); column in c.
__device__ __forceinline__ int half_row(uint32_t pos, const BlockGeom &g, uint32_t &c)
{
    uint32_t r;
    split_pos(pos, g, r, c);
    return (int)(2u * r + (c >= (uint32_t)kHalf ? 1u : 0u));
}

// Decoder wavefront d of kWideDecoders: the chunks cb0 + d, cb0 + d + kWideDecoders, ...
// of block b into list / hp (Algorithm 2 steps 5-9, the "arrange" of step 9 being the
// list order).  Every one of the kHalfKeys + 1 pointers is written for every block:
// by the entry that starts a half row (for all half rows since the entry before it,
// whichever chunk that was in - its position is this entry's minus the gap), and
// after the block's last entry up to the end by the wavefront that decodes the last
// chunk; a block without entries gets all pointers zero from decoder 0.
__device__ __forceinline__ void wide_decode_block(const LayerDev &L, const Tables &T, uint32_t b, int d, int lane,
                                                  uint16_t *list, uint16_t *hp, int cap)
{
    const uint32_t cb0 = L.block_chunk[b], cb1 = L.block_chunk[b + 1];
    if (cb0 == cb1) {
        if (d == 0)
            for (int k = lane; k <= kHalfKeys; k += 64) hp[k] = 0;
        return;
    }
    const BlockGeom g = block_geom(L, b);
    const uint32_t nz0 = L.chunk_nz[cb0];
    // one chunk ahead: the head and record of the next chunk are requested before this one is decoded
    uint32_t c = cb0 + (uint32_t)d;
    ChunkHead h{};
    LaneRecord rec{};
    uint32_t nzc = 0;
    if (c < cb1) {
        h = load_head(L, c);
        rec = load_record(L, h, lane);
        nzc = L.chunk_nz[c];
    }
    while (c < cb1) {
        const uint32_t cn = c + (uint32_t)kWideDecoders;
        ChunkHead hn{};
        LaneRecord recn{};
        uint32_t nzn = 0;
        if (cn < cb1) {
            hn = load_head(L, cn);
            recn = load_record(L, hn, lane);
            nzn = L.chunk_nz[cn];
        }
        const Symbols y = decode_record(rec, T);
        // entries of the lane that are not padding; with the lane's advance in one scan
        uint32_t nzl = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) nzl = __builtin_amdgcn_sad_u8(nonzero_bytes(y.v[w]), 0u, nzl);
        const uint32_t mine = nzl | (y.adv << 10);
        const uint32_t incl = wave_incl_scan(mine);
        uint32_t rank = nzc - nz0 + ((incl - mine) & 1023u);
        const uint32_t sum = h.m.pos0 + ((incl - mine) >> 10);
        // half row of the entry before the lane's first (none before the block's first)
        uint32_t cc;
        int pkey = sum == 0u ? -1 : half_row(sum - 1u, g, cc);
        for_each_entry(y, sum, [&](uint32_t, uint32_t v, uint32_t, uint32_t pos) {
            const int key = half_row(pos, g, cc);
            for (int k = pkey + 1; k <= key; ++k) hp[k] = (uint16_t)rank;
            pkey = key;
            if (v != 0u) {
                list[min(rank, (uint32_t)cap - 1u)] = (uint16_t)((cc << 8) | v);
                ++rank;
            }
        });
        if (c + 1u == cb1) {
            // the block's last chunk: the half rows after its last entry start at the end of the list
            const uint32_t total = nzc - nz0 + ((uint32_t)__builtin_amdgcn_readlane((int)incl, 63) & 1023u);
            const int klast = (int)wave_max((uint32_t)(y.n ? pkey : 0));
            for (int k = klast + 1 + lane; k <= kHalfKeys; k += 64) hp[k] = (uint16_t)total;
        }
        c = cn;
        h = hn;
        rec = recn;
        nzc = nzn;
    }
}

// IPL consecutive floats from LDS / to LDS / from global memory with one access.
template <int IPL> struct WideVec {
    typedef float type __attribute__((ext_vector_type(IPL)));
};
template <> struct WideVec<1> {
    typedef float type;
};

template <int IPL>
__global__ __launch_bounds__(kWideThreads) void fc_wide_kernel(LayerDev L, const float *__restrict__ XT, float *part, int panels,
                                                               int splits, int Bp, int cap)
{
    typedef typename WideVec<IPL>::type vec_t;
    constexpr int kImages = 64 * IPL;
    constexpr int kBatch = 4;                                         // entries whose activations are requested together
    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    const Smem s = carve(smem_raw, L);
    uint16_t *hp = (uint16_t *)s.extra;                                 // [2][kHalfPtrStride]
    uint16_t *lists = hp + 2 * kHalfPtrStride;                          // [2][cap]
    float *slabs = (float *)(lists + 2 * (size_t)cap);                  // [2][kHalf][kImages]
    // consecutive workgroups take the splits of one block row: with the usual eight
    // splits the workgroups that share a range of activation rows share a die's L2
    const int j = (int)blockIdx.x % splits, rest = (int)blockIdx.x / splits;
    const int p = rest % panels, nb = rest / panels;
    const int pj = p * splits + j;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    const int blk_lo = (int)(((int64_t)L.nbw * j) / splits), blk_hi = (int)(((int64_t)L.nbw * (j + 1)) / splits);
    const uint32_t pb0 = (uint32_t)p * (uint32_t)L.nbw;
    const int nh = L.bw > kHalf ? 2 : 1;
    const int phases = (blk_hi - blk_lo) * nh;
    const bool decoder = wave >= kWideMults;

    // a wavefront's share of a slab: rows 4 wave .. 4 wave + 3, IPL floats per lane and row
    const float *xsrc = XT + (size_t)nb * kImages + (size_t)lane * IPL;
    auto slab_row0 = [&](int ph) { return (size_t)(blk_lo + ph / nh) * kTile + (size_t)(ph % nh) * kHalf; };
    // (a multiplying wavefront, short of registers, takes its rows in two halves: one during
    // each half of its phase)
    vec_t stage[kSlabRowsPerWave];
    auto slab_fetch = [&](int ph, int q0, int q1) {
        const float *src = xsrc + (slab_row0(ph) + (size_t)wave * kSlabRowsPerWave) * (size_t)Bp;
#pragma unroll
        for (int q = q0; q < q1; ++q) stage[q] = *(const vec_t *)(src + (size_t)q * Bp);
    };
    auto slab_store = [&](int ph, int q0, int q1) {
        float *dst = slabs + (size_t)(ph & 1) * kHalf * kImages + (size_t)(wave * kSlabRowsPerWave) * kImages + lane * IPL;
#pragma unroll
        for (int q = q0; q < q1; ++q) *(vec_t *)(dst + q * kImages) = stage[q];
    };
    constexpr int kStageHalf = kSlabRowsPerWave / 2;

    if (phases > 0) slab_fetch(0, 0, kSlabRowsPerWave);
    if (threadIdx.x < kThreads) store_tables(s, L, fetch_tables(L));
    if (phases > 0) slab_store(0, 0, kSlabRowsPerWave);
    if (decoder) {
        // The decoders' side of every barrier below, in a loop of their own: a shared loop
        // would keep the multipliers' sums alive in the decoders' registers.
        __builtin_amdgcn_s_setprio(3);
        __syncthreads();                                    // tables stored
        if (phases > 0) wide_decode_block(L, s.T, pb0 + (uint32_t)blk_lo, wave - kWideMults, lane, lists, hp, cap);
        __syncthreads();                                    // first block's list, first slab
        for (int ph = 0; ph < phases; ++ph) {
            const int i = ph / nh, h = ph - i * nh;
            const bool more = ph + 1 < phases;
            if (more) slab_fetch(ph + 1, 0, kSlabRowsPerWave);
            if (h == 0 && i + 1 < blk_hi - blk_lo)
                wide_decode_block(L, s.T, pb0 + (uint32_t)(blk_lo + i + 1), wave - kWideMults, lane,
                                  lists + (size_t)((i + 1) & 1) * cap, hp + ((i + 1) & 1) * kHalfPtrStride, cap);
            if (more) slab_store(ph + 1, 0, kSlabRowsPerWave);
            __syncthreads();
        }
        return;
    }

    float acc[kWideRows][IPL];
#pragma unroll
    for (int r = 0; r < kWideRows; ++r)
#pragma unroll
        for (int q = 0; q < IPL; ++q) acc[r][q] = 0.0f;
    __syncthreads();                                        // tables stored
    __syncthreads();                                        // first block's list, first slab
    uint32_t hpv = 0;                                       // the wavefront's half-row pointers, one per lane
    for (int ph = 0; ph < phases; ++ph) {
        const int i = ph / nh, h = ph - i * nh;
        const bool more = ph + 1 < phases;
        {
            if (more) slab_fetch(ph + 1, 0, kStageHalf);
            const uint16_t *list = lists + (size_t)(i & 1) * cap;
            const float *slab = slabs + (size_t)(ph & 1) * kHalf * kImages + lane * IPL;
            if (h == 0) hpv = hp[(i & 1) * kHalfPtrStride + min(2 * kWideRows * wave + lane, kHalfKeys)];
            // the rows in two groups: the entries of a group's rows in this phase, one per lane, and
            // their weights are fetched together, then the rows are walked one after the other
            constexpr int kGroup = (kWideRows + 1) / 2;
#pragma unroll
            for (int r0 = 0; r0 < kWideRows; r0 += kGroup) {
                if (r0 > 0 && more) {
                    slab_store(ph + 1, 0, kStageHalf);
                    slab_fetch(ph + 1, kStageHalf, kSlabRowsPerWave);
                }
                uint32_t ev[kGroup];
                float wv[kGroup];
                int cnt[kGroup];
#pragma unroll
                for (int g = 0; g < kGroup; ++g) {
                    const int r = r0 + g;
                    if (r >= kWideRows) break;
                    const int a = __builtin_amdgcn_readlane((int)hpv, 2 * r + h), e = __builtin_amdgcn_readlane((int)hpv, 2 * r + h + 1);
                    cnt[g] = e - a;
                    ev[g] = lane < cnt[g] ? (uint32_t)list[min(a + lane, cap - 1)] : 0u;
                }
#pragma unroll
                for (int g = 0; g < kGroup; ++g)
                    if (r0 + g < kWideRows) wv[g] = s.T.cb[ev[g] & 0xffu];
#pragma unroll
                for (int g = 0; g < kGroup; ++g) {
                    const int r = r0 + g;
                    if (r >= kWideRows) break;
                    const int n = cnt[g];
                    auto one = [&](int jj, vec_t &x, float &w) {
                        const uint32_t se = (uint32_t)__builtin_amdgcn_readlane((int)ev[g], jj);
                        w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wv[g]), jj));
                        x = *(const vec_t *)(slab + ((se >> 8) & (uint32_t)(kHalf - 1)) * kImages);
                    };
                    auto fma = [&](const vec_t &x, float w) {
                        if constexpr (IPL == 1) acc[r][0] += w * x;
                        else {
#pragma unroll
                            for (int q = 0; q < IPL; ++q) acc[r][q] += w * x[q];
                        }
                    };
                    int jj = 0;
                    if constexpr (kBatch == 8) {
                        // the first eight entries in one piece without a branch: a slot past the row's
                        // last entry takes that entry's activations again with weight 0
                        if (n > 0) {
                            vec_t x[8];
                            float w[8];
#pragma unroll
                            for (int u = 0; u < 8; ++u) {
                                one(min(u, n - 1), x[u], w[u]);
                                w[u] = u < n ? w[u] : 0.0f;
                            }
#pragma unroll
                            for (int u = 0; u < 8; ++u) fma(x[u], w[u]);
                        }
                        for (jj = 8; jj < n; ++jj) {
                            vec_t x;
                            float w;
                            one(jj, x, w);
                            fma(x, w);
                        }
                        continue;
                    } else {
                        for (; jj + 4 <= n; jj += 4) {
                            vec_t x[4];
                            float w[4];
#pragma unroll
                            for (int u = 0; u < 4; ++u) one(jj + u, x[u], w[u]);
#pragma unroll
                            for (int u = 0; u < 4; ++u) fma(x[u], w[u]);
                        }
                    }
                    if (n & 2) {
                        vec_t x[2];
                        float w[2];
#pragma unroll
                        for (int u = 0; u < 2; ++u) one(jj + u, x[u], w[u]);
#pragma unroll
                        for (int u = 0; u < 2; ++u) fma(x[u], w[u]);
                        jj += 2;
                    }
                    if (n & 1) {
                        vec_t x;
                        float w;
                        one(jj, x, w);
                        fma(x, w);
                    }
                }
            }
            if (more) slab_store(ph + 1, kStageHalf, kSlabRowsPerWave);
        }
        __syncthreads();
    }
    // the wavefront's rows of the workgroup's partial tile, part[pj][row][Bp]: a row's images are contiguous
    float *mine = part + ((size_t)pj * kTile + (size_t)wave * kWideRows) * (size_t)Bp + (size_t)nb * kImages + (size_t)lane * IPL;
#pragma unroll
    for (int r = 0; r < kWideRows; ++r) {
        if (wave * kWideRows + r >= kTile) break;
        vec_t v;
        if constexpr (IPL == 1) v = acc[r][0];
        else {
#pragma unroll
            for (int q = 0; q < IPL; ++q) v[q] = acc[r][q];
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
