// Fixed-function layers of a whole network (Table IV: pool, norm).
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

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

// One thread per (image, run of kLrnChunk channels, pixel): consecutive threads take
// consecutive pixels, so every load and store of a wavefront is one contiguous run.
// HALF = n / 2 for the usual small windows: the run and its neighbours are loaded once
// and a channel's window is summed from registers, in channel order; HALF < 0: any
// window, summed from the (cached) input as it stands.
// (One thread per pixel walking all channels took 214 us for one image of 256 x 27 x 27.)
constexpr int kLrnChunk = 4;

template <int HALF>
__global__ __launch_bounds__(256) void lrn_kernel(const float *__restrict__ X, float *Y, int B, int C, int64_t hw, int n,
                                                  float alpha_over_n, float beta, float k)
{
    // blockIdx.x: 256 pixels; blockIdx.y, strided: (image, run of channels) - uniform per workgroup
    const int half = n / 2;
    const int n_chunks = (C + kLrnChunk - 1) / kLrnChunk;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= hw) return;
    for (int bc = (int)blockIdx.y; bc < B * n_chunks; bc += (int)gridDim.y) {
        const int c0 = (bc % n_chunks) * kLrnChunk;
        const int64_t b = bc / n_chunks;
        const float *x = X + b * C * hw + i;
        float *y = Y + b * C * hw + i;
        if (HALF >= 0) {
            float v[kLrnChunk + 2 * (HALF >= 0 ? HALF : 0)];
#pragma unroll
            for (int j = 0; j < kLrnChunk + 2 * HALF; ++j) {
                const int cc = c0 - HALF + j;
                v[j] = cc >= 0 && cc < C ? x[(int64_t)cc * hw] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < kLrnChunk; ++j) {
                float ss = 0.0f;
#pragma unroll
                for (int w = 0; w <= 2 * HALF; ++w) ss += v[j + w] * v[j + w];
                if (c0 + j < C) y[(int64_t)(c0 + j) * hw] = v[j + HALF] * powf(k + alpha_over_n * ss, -beta);
            }
        } else {
            for (int c = c0; c < min(C, c0 + kLrnChunk); ++c) {
                float ss = 0.0f;
                for (int cc = max(0, c - half); cc <= min(C - 1, c + half); ++cc) {
                    const float v = x[(int64_t)cc * hw];
                    ss += v * v;
                }
                y[(int64_t)c * hw] = x[(int64_t)c * hw] * powf(k + alpha_over_n * ss, -beta);
            }
        }
    }
}
