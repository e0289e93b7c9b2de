// Row-wise pieces of the target pass: embedding gather, RMSNorm, rotary tables.
#pragma once
#include "duo_common.h"
#include "duo_gemm.h"

// x[m] = E[token_m], plus what the first RMSNorm needs (see RowScale in duo_gemm.h): u = x * gain as
// bf16 pairs in the QKV projection's operand buffer and the per-tile partial sums of x^2.  Also the
// device-side input checks: token ids in range, device prefix length equal to the host's.
// One workgroup (256 threads) per row; a thread handles runs of eight consecutive channels.
__global__ __launch_bounds__(256) void embed_kernel(const u16* __restrict__ embed, const int32_t* __restrict__ tokens,
                                                     int root_token, RowPlan plan, int vocab, const int32_t* prefix_len,
                                                     int32_t* status, float* __restrict__ x, const u16* __restrict__ gain,
                                                     u16* __restrict__ h, int d, int pair_rows, int tiles,
                                                     float* __restrict__ ssq_part) {
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
    for (int j8 = threadIdx.x * 8; j8 < d; j8 += 256 * 8) {
        Frag8 ev, gv, hi, lo;
        ev.q = *reinterpret_cast<const u32x4*>(e + j8);
        gv.q = *reinterpret_cast<const u32x4*>(gain + j8);
        float sq = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float xv = bf16_to_f32(ev.h[j]);
            xr[j8 + j] = xv;
            sq += xv * xv;
            const float u = xv * bf16_to_f32(gv.h[j]);
            hi.h[j] = f32_to_bf16(u);
            lo.h[j] = f32_to_bf16(u - bf16_to_f32(hi.h[j]));
        }
        *reinterpret_cast<u32x4*>(h + operand_offset(m, j8, tiles)) = hi.q;
        *reinterpret_cast<u32x4*>(h + operand_offset(pair_rows + m, j8, tiles)) = lo.q;
        sq += __shfl_xor(sq, 1, 64);  // two runs of eight = one 16-column tile
        if (!(threadIdx.x & 1)) ssq_part[(size_t)m * (d >> 4) + (j8 >> 4)] = sq;
    }
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
