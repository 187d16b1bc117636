// Finishing kernel of the dense-tile paths (sum of the splits, bias, activation, output layout).
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

// Finishes the dense-tile path: Y = act(sum over the splits of a block row, in a fixed
// order, + bias) (Eq. 1).  A workgroup takes a block row and ct <= kColTile consecutive
// columns (images, or image x output pixel for a convolution): for each split that
// is one contiguous run of ct x bh floats of the partial buffer.  The host picks ct
// so that the launch still has a few workgroups per CU.  FC output
// rows are contiguous in Y[image][row]; a convolution's output is contiguous along
// the pixels, Y[image][row][pixel], so its tile is turned in LDS first.  The same
// turned form with conv_pq = the padded image count of a following layer writes the
// output as that layer's transposed activations, XT[row][image]; columns from ncols up
// to zero_to are then written as zeros (the padded images of that layout).  The rows of
// a block row can be shared out among workgroups, rt to each (the host's choice, as ct).
constexpr int kColTile = 32;

__global__ __launch_bounds__(256) void mfma_reduce_kernel(LayerDev L, const float *__restrict__ part,
                                                          const float *__restrict__ bias, float *Y, int ncols, int part_b,
                                                          int splits, int relu, int conv_pq, int ct, int zero_to, int rt)
{
    __shared__ float tile[kColTile][kTile + 1];
    // workgroup -> (block row, column tile, row tile of rt rows)
    const int ntile = (max(ncols, zero_to) + ct - 1) / ct, nrt = (L.bh + rt - 1) / rt;
    const int pl = (int)blockIdx.x / (ntile * nrt), rem = (int)blockIdx.x - pl * ntile * nrt;
    const int p = L.panel0 + pl;                            // part slots are numbered from the launch's first block row
    const int c0 = (rem / nrt) * ct, r0 = (rem % nrt) * rt;
    const int row_id = p * L.bh;
    const int bhp = min(L.bh, L.M - row_id);
    const int r1 = min(r0 + rt, bhp);                       // this workgroup's rows are r0 .. r1 - 1
    const size_t split_stride = (size_t)part_b * L.bh;
    for (int e = threadIdx.x; e < ct * rt; e += blockDim.x) {
        const int ci = e / rt, r = r0 + (e - ci * rt);
        const int c = c0 + ci;
        if (r >= r1) continue;
        if (c >= ncols) {
            if (conv_pq != 0) tile[ci][r] = 0.0f;
            continue;
        }
        const float *src = part + ((size_t)pl * splits * part_b + c) * L.bh + r;
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
    for (int e = threadIdx.x; e < ct * (r1 - r0); e += blockDim.x) {
        const int r = r0 + e / ct, ci = e % ct;
        const int c = c0 + ci;
        if (c < max(ncols, zero_to)) Y[((size_t)(c / conv_pq) * L.M + row_id + r) * conv_pq + (c % conv_pq)] = tile[ci][r];
    }
}
