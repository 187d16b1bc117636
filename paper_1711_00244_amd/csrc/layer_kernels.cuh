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
// consecutive pixels, so every load and store of a wavefront is one contiguous run; a
// channel's window is summed from the (cached) input as it stands, in channel order.
// (One thread per pixel walking all channels took 214 us for one image of 256 x 27 x 27.)
constexpr int kLrnChunk = 4;

__global__ __launch_bounds__(256) void lrn_kernel(const float *__restrict__ X, float *Y, int B, int C, int64_t hw, int n,
                                                  float alpha_over_n, float beta, float k)
{
    const int half = n / 2;
    const int n_chunks = (C + kLrnChunk - 1) / kLrnChunk;
    const int64_t total = (int64_t)B * n_chunks * hw;
    for (int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i = t % hw, bc = t / hw;
        const int chunk = (int)(bc % n_chunks);
        const int64_t b = bc / n_chunks;
        const float *x = X + b * C * hw + i;
        float *y = Y + b * C * hw + i;
        for (int c = chunk * kLrnChunk; c < min(C, (chunk + 1) * kLrnChunk); ++c) {
            float ss = 0.0f;
            for (int cc = max(0, c - half); cc <= min(C - 1, c + half); ++cc) {
                const float v = x[(int64_t)cc * hw];
                ss += v * v;
            }
            y[(int64_t)c * hw] = x[(int64_t)c * hw] * powf(k + alpha_over_n * ss, -beta);
        }
    }
}
