// Fixed-function layers of a whole network (Table IV: pool, norm).
// Part of the device translation unit: included by device.hip inside namespace cl,
// in the order given there.
#pragma once

// One thread per output.  A row of workgroups (blockIdx.y, strided) takes planes_per_row
// whole (image, channel) planes - as many as give it about 2048 outputs, so that small
// planes still fill the workgroups - and blockIdx.x with the thread gives the plane within
// the row and the output's place in it with two 32-bit divisions.  SIZE: the window when it
// is 2 or 3 (its loads are then all in flight together), 0: any window.
// (Taking image, channel, row and column from one flat 64-bit index cost three 64-bit
// divisions per output: 38 us for 64 x 96 x 55 x 55, where the copy rate allows 13.)
template <int SIZE>
__global__ __launch_bounds__(256) void maxpool_kernel(const float *__restrict__ X, float *Y, int64_t planes, int H, int W,
                                                      int P, int Q, int size, int stride, int planes_per_row)
{
    const unsigned pq = (unsigned)P * (unsigned)Q;
    const unsigned t = blockIdx.x * 256u + threadIdx.x;
    const unsigned lp = t / pq, i = t - lp * pq;
    if (lp >= (unsigned)planes_per_row) return;
    const unsigned p = i / (unsigned)Q, q = i - p * (unsigned)Q;
    const int64_t in_off = ((int64_t)p * W + q) * stride, hw = (int64_t)H * W;
    const int sz = SIZE ? SIZE : size;
    for (int64_t pl = (int64_t)blockIdx.y * planes_per_row + lp; pl < planes; pl += (int64_t)gridDim.y * planes_per_row) {
        const float *x = X + pl * hw + in_off;
        float m = x[0];
#pragma unroll
        for (int r = 0; r < sz; ++r)
#pragma unroll
            for (int s = 0; s < sz; ++s) m = fmaxf(m, x[(int64_t)r * W + s]);
        Y[pl * pq + i] = m;
    }
}

// One thread per (image, run of kLrnChunk channels, pixel): consecutive threads take
// consecutive pixels, so every load and store of a wavefront is one contiguous run.
// HALF = n / 2 for the usual small windows: the run and its neighbours are loaded once
// and a channel's window is summed from registers, in channel order; HALF < 0: any
// window, summed from the (cached) input as it stands.
// (One thread per pixel walking all channels took 214 us for one image of 256 x 27 x 27.)
constexpr int kLrnChunk = 8;

// base^(-beta).  For a positive, normal, finite base: exp2(-beta * log2(base)) with the
// two hardware instructions (v_log_f32, v_exp_f32), whose error of about one unit in the
// last place each leaves a relative error near 1e-7 * (1 + |beta * log2(base)|) in the
// result; any other base goes through the library's powf, which alone took 120
// instructions per element and made the kernel ALU-bound (67 us for 64 x 96 x 55 x 55,
// three times a copy).
__device__ __forceinline__ float pow_neg(float base, float beta)
{
    if (!(base >= 1.17549435e-38f && base <= 3.0e38f)) return powf(base, -beta);
    return __builtin_amdgcn_exp2f(-beta * __builtin_amdgcn_logf(base));
}

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
                if (c0 + j < C) y[(int64_t)(c0 + j) * hw] = v[j + HALF] * pow_neg(k + alpha_over_n * ss, beta);
            }
        } else {
            for (int c = c0; c < min(C, c0 + kLrnChunk); ++c) {
                float ss = 0.0f;
                for (int cc = max(0, c - half); cc <= min(C - 1, c + half); ++cc) {
                    const float v = x[(int64_t)cc * hw];
                    ss += v * v;
                }
                y[(int64_t)c * hw] = x[(int64_t)c * hw] * pow_neg(k + alpha_over_n * ss, beta);
            }
        }
    }
}
