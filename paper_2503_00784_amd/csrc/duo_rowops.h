// Row-wise pieces of the target pass: embedding gather, RMSNorm, rotary tables.
#pragma once
#include "duo_common.h"
#include "duo_gemm.h"

__device__ __forceinline__ float block_sum_256(float v, float* sm) {
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) sm[wave] = v;
    __syncthreads();
    const float t = sm[0] + sm[1] + sm[2] + sm[3];
    __syncthreads();
    return t;
}

// h[m] = x[m] * rsqrt(mean(x[m]^2) + eps) * gain as a bf16 pair, written into a GEMM operand buffer
// (tile order, see duo_gemm.h): hi as operand row m, lo as operand row m + pair_rows.  One workgroup
// (256 threads) per row; a thread handles runs of eight consecutive channels = one 16-byte store.
__device__ __forceinline__ void rmsnorm_row(const float* __restrict__ xr, const u16* __restrict__ gain,
                                            u16* __restrict__ h, int m, int pair_rows, int tiles, int d, float eps,
                                            float* sm) {
    float ss = 0.f;
    for (int j = threadIdx.x; j < d; j += 256) {
        const float v = xr[j];
        ss += v * v;
    }
    const float tot = block_sum_256(ss, sm);
    const float rs = 1.0f / sqrtf(tot / (float)d + eps);
    for (int j8 = threadIdx.x * 8; j8 < d; j8 += 256 * 8) {
        Frag8 hi, lo;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float v = xr[j8 + j] * rs * bf16_to_f32(gain[j8 + j]);
            hi.h[j] = f32_to_bf16(v);
            lo.h[j] = f32_to_bf16(v - bf16_to_f32(hi.h[j]));
        }
        *reinterpret_cast<u32x4*>(h + operand_offset(m, j8, tiles)) = hi.q;
        *reinterpret_cast<u32x4*>(h + operand_offset(pair_rows + m, j8, tiles)) = lo.q;
    }
}

__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, const u16* __restrict__ gain,
                                                       u16* __restrict__ h, int d, int pair_rows, int tiles, float eps) {
    __shared__ float sm[4];
    const int m = blockIdx.x;
    rmsnorm_row(x + (size_t)m * d, gain, h, m, pair_rows, tiles, d, eps, sm);
}

// x[m] = E[token_m]; h[m] = RMSNorm(x[m]) with the first layer's gain.  Also the device-side
// input checks: token ids in range, device prefix length equal to the host's.
__global__ __launch_bounds__(256) void embed_norm_kernel(const u16* __restrict__ embed, const int32_t* __restrict__ tokens,
                                                          int root_token, RowPlan plan, int vocab, const int32_t* prefix_len,
                                                          int32_t* status, float* __restrict__ x, const u16* __restrict__ gain,
                                                          u16* __restrict__ h, int d, int pair_rows, int tiles, float eps) {
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
    rmsnorm_row(xr, gain, h, m, pair_rows, tiles, d, eps, sm);
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
