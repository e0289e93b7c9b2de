// Row-wise pieces of the target pass: embedding gather, RMSNorm, rotary tables.
#pragma once
#include "duo_common.h"

__device__ __forceinline__ float block_sum_256(float v, float* sm) {
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) sm[wave] = v;
    __syncthreads();
    const float t = sm[0] + sm[1] + sm[2] + sm[3];
    __syncthreads();
    return t;
}

// h[m] = x[m] * rsqrt(mean(x[m]^2) + eps) * gain as a bf16 pair: hi in row m, lo in row m + pair_rows
// of the GEMM operand buffer.  One workgroup (256 threads) per row.
__device__ __forceinline__ void rmsnorm_row(const float* __restrict__ xr, const u16* __restrict__ gain,
                                            u16* __restrict__ hi_row, u16* __restrict__ lo_row, int d, float eps,
                                            float* sm) {
    float ss = 0.f;
    for (int j = threadIdx.x; j < d; j += 256) {
        const float v = xr[j];
        ss += v * v;
    }
    const float tot = block_sum_256(ss, sm);
    const float rs = 1.0f / sqrtf(tot / (float)d + eps);
    for (int j = threadIdx.x; j < d; j += 256) {
        const float h = xr[j] * rs * bf16_to_f32(gain[j]);
        const u16 hi = f32_to_bf16(h);
        hi_row[j] = hi;
        lo_row[j] = f32_to_bf16(h - bf16_to_f32(hi));
    }
}

__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, const u16* __restrict__ gain,
                                                       u16* __restrict__ h, int d, int pair_rows, float eps) {
    __shared__ float sm[4];
    const int m = blockIdx.x;
    rmsnorm_row(x + (size_t)m * d, gain, h + (size_t)m * d, h + (size_t)(pair_rows + m) * d, d, eps, sm);
}

// x[m] = E[token_m]; h[m] = RMSNorm(x[m]) with the first layer's gain.  Also the device-side
// input checks: token ids in range, device prefix length equal to the host's.
__global__ __launch_bounds__(256) void embed_norm_kernel(const u16* __restrict__ embed, const int32_t* __restrict__ tokens,
                                                          int root_token, RowPlan plan, int vocab, const int32_t* prefix_len,
                                                          int32_t* status, float* __restrict__ x, const u16* __restrict__ gain,
                                                          u16* __restrict__ h, int d, int pair_rows, float eps) {
    __shared__ float sm[4];
    const int m = blockIdx.x;
    if (m == 0 && threadIdx.x == 0 && prefix_len && status && *prefix_len != plan.P)
        atomicOr(status, 2);
    int tok = m < plan.R ? root_token : tokens[m - plan.R];
    if (tok < 0 || tok >= vocab) {
        if (threadIdx.x == 0 && status) atomicOr(status, 1);
        tok = tok < 0 ? 0 : vocab - 1;
    }
    const u16* e = embed + (size_t)tok * d;
    float* xr = x + (size_t)m * d;
    for (int j = threadIdx.x; j < d; j += 256) xr[j] = bf16_to_f32(e[j]);
    __syncthreads();
    rmsnorm_row(xr, gain, h + (size_t)m * d, h + (size_t)(pair_rows + m) * d, d, eps, sm);
}

// cos/sin of pos(m) * theta^(-2d/D), evaluated in double and rounded once to fp32.
__global__ void rope_table_kernel(RowPlan plan, int D, double theta, float* __restrict__ rc, float* __restrict__ rs) {
    const int m = blockIdx.x, half = D / 2;
    if (m >= plan.M) return;
    for (int d = threadIdx.x; d < half; d += blockDim.x) {
        const double ang = (double)plan.pos(m) * pow(theta, -2.0 * (double)d / (double)D);
        rc[m * half + d] = (float)cos(ang);
        rs[m * half + d] = (float)sin(ang);
    }
}

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
