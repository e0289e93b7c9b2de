// Row-wise pieces of the target pass: embedding gather, RMSNorm, rotary tables.
#pragma once
#include "duo_common.h"
#include "duo_gemm.h"
#include "duo_sample.h"

// Sum of `v` over the NWV * 64 threads of a workgroup in a fixed order (lanes by butterfly, then the waves
// in index order); thread 0 stores it.
template <int NWV>
__device__ __forceinline__ void block_row_sum(float v, float* wsum, float* out) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = wsum[0];
#pragma unroll
        for (int w = 1; w < NWV; ++w) t += wsum[w];
        *out = t;
    }
}

// x[m] = E[token_m], plus what the first RMSNorm needs (see RowScale in duo_gemm.h): u = x * gain as
// bf16 pairs in the QKV projection's operand buffer and the per-tile partial sums of x^2.  Also the
// device-side input checks: token ids in range, device prefix length equal to the host's.
// One workgroup (256 threads) per row; a thread handles runs of eight consecutive channels.
__global__ __launch_bounds__(256) void embed_kernel(const u16* __restrict__ embed, const int32_t* __restrict__ tokens,
                                                     int root_token, RowPlan plan, int vocab, const int32_t* prefix_len,
                                                     int32_t* status, float* __restrict__ x, const u16* __restrict__ gain,
                                                     u16* __restrict__ h, int d, int pair_rows, int tiles,
                                                     float* __restrict__ ssq_part, float* __restrict__ ssq_full) {
    __shared__ float wsum[4];
    const int m = blockIdx.x;
    float total = 0.f;
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
            const float xv = elem_to_f32(ev.h[j]);
            xr[j8 + j] = xv;
            sq += xv * xv;
            const float u = xv * elem_to_f32(gv.h[j]);
            hi.h[j] = f32_to_elem(u);
            lo.h[j] = f32_to_elem(u - elem_to_f32(hi.h[j]));
        }
        *reinterpret_cast<u32x4*>(h + operand_offset(m, j8, tiles)) = hi.q;
        *reinterpret_cast<u32x4*>(h + operand_offset(pair_rows + m, j8, tiles)) = lo.q;
        total += sq;
        sq += __shfl_xor(sq, 1, 64);  // two runs of eight = one 16-column tile
        if (!(threadIdx.x & 1)) ssq_part[(size_t)m * (d >> 4) + (j8 >> 4)] = sq;
    }
    block_row_sum<4>(total, wsum, ssq_full + (size_t)m * RowScale::FULL_PARTS);  // one range: the whole row
    if (threadIdx.x >= 1 && threadIdx.x < RowScale::FULL_PARTS) ssq_full[(size_t)m * RowScale::FULL_PARTS + threadIdx.x] = 0.f;
}

// Second half of a residual projection whose K range was split over workgroups: x[m] += sum of the S
// partial results (added in split order), then what EpiResidual does for the next RMSNorm: u = x * gain
// as bf16 pairs in operand layout and the partial sums of x^2 per 16-column tile, plus the sum of squares over this
// workgroup's whole column range (RowScale::full), which the consumer reads instead of 256 partials per row.
// grid = (rows, P): workgroup (m, pt) takes columns pt * d/P .. of row m (d/P a multiple of 64; P <= FULL_PARTS),
// NWV waves, eight consecutive channels per thread and turn; the loads of all
// splits are issued together (S <= 8, indices beyond S re-read the last split and are not added).
template <int NWV>
__global__ __launch_bounds__(NWV * 64) void residual_reduce_kernel(const float* __restrict__ part, int S, size_t split_stride,
                                                                   float* __restrict__ x, const u16* __restrict__ gain,
                                                                   u16* __restrict__ h, int d, int pair_rows, int tiles,
                                                                   float* __restrict__ ssq_part, float* __restrict__ ssq_full) {
    __shared__ float wsum[NWV];
    const int m = blockIdx.x, P = gridDim.y, cols = d / P, c0 = blockIdx.y * cols;
    float total = 0.f;
    for (int j8 = c0 + threadIdx.x * 8; j8 < c0 + cols; j8 += NWV * 64 * 8) {  // lanes leave in pairs
        float* xr = x + (size_t)m * d + j8;
        const float* pr = part + (size_t)m * d + j8;
        f32x4 p0[8], p1[8];
#pragma unroll
        for (int sp = 0; sp < 8; ++sp) {
            const float* ps = pr + (size_t)(sp < S ? sp : S - 1) * split_stride;
            p0[sp] = *reinterpret_cast<const f32x4*>(ps);
            p1[sp] = *reinterpret_cast<const f32x4*>(ps + 4);
        }
        f32x4 a0 = *reinterpret_cast<const f32x4*>(xr), a1 = *reinterpret_cast<const f32x4*>(xr + 4);
        Frag8 gv, hi, lo;
        gv.q = *reinterpret_cast<const u32x4*>(gain + j8);
#pragma unroll
        for (int sp = 0; sp < 8; ++sp) {
            if (sp < S) {
                a0 += p0[sp];
                a1 += p1[sp];
            }
        }
        *reinterpret_cast<f32x4*>(xr) = a0;
        *reinterpret_cast<f32x4*>(xr + 4) = a1;
        float sq = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float xv = j < 4 ? a0[j] : a1[j - 4];
            sq += xv * xv;
            const float u = xv * elem_to_f32(gv.h[j]);
            hi.h[j] = f32_to_elem(u);
            lo.h[j] = f32_to_elem(u - elem_to_f32(hi.h[j]));
        }
        *reinterpret_cast<u32x4*>(h + operand_offset(m, j8, tiles)) = hi.q;
        *reinterpret_cast<u32x4*>(h + operand_offset(pair_rows + m, j8, tiles)) = lo.q;
        total += sq;
        sq += __shfl_xor(sq, 1, 64);
        if (!(threadIdx.x & 1)) ssq_part[(size_t)m * (d >> 4) + (j8 >> 4)] = sq;
    }
    block_row_sum<NWV>(total, wsum, ssq_full + (size_t)m * RowScale::FULL_PARTS + blockIdx.y);
    if (blockIdx.y == 0 && (int)threadIdx.x >= P && threadIdx.x < RowScale::FULL_PARTS)
        ssq_full[(size_t)m * RowScale::FULL_PARTS + threadIdx.x] = 0.f;  // unused ranges
}

// Column ranges per row for residual_reduce_kernel: enough workgroups to fill the chip when there are few rows.
static inline int reduce_parts(int M, int d) {
    int P = M <= 32 ? 8 : (M <= 80 ? 4 : (M < 256 ? 2 : 1));
    while (P > 1 && d % (P * 64) != 0) P >>= 1;
    return P;
}
static inline void launch_residual_reduce(int M, const float* part, int S, size_t split_stride, float* x, const u16* gain,
                                          u16* h, int d, int pair_rows, int tiles, float* ssq_part, float* ssq_full,
                                          hipStream_t s) {
    const int P = reduce_parts(M, d), cols = d / P;
    const dim3 grid(M, P);
    if (cols <= 512) DUO_LAUNCH(residual_reduce_kernel<1>, grid, dim3(64), s, part, S, split_stride, x, gain, h, d, pair_rows, tiles, ssq_part, ssq_full);
    else if (cols <= 1024) DUO_LAUNCH(residual_reduce_kernel<2>, grid, dim3(128), s, part, S, split_stride, x, gain, h, d, pair_rows, tiles, ssq_part, ssq_full);
    else if (cols <= 2048) DUO_LAUNCH(residual_reduce_kernel<4>, grid, dim3(256), s, part, S, split_stride, x, gain, h, d, pair_rows, tiles, ssq_part, ssq_full);
    else DUO_LAUNCH(residual_reduce_kernel<8>, grid, dim3(512), s, part, S, split_stride, x, gain, h, d, pair_rows, tiles, ssq_part, ssq_full);
}

// Second half of a Q/K/V projection whose K range was split over workgroups (64 rows and more: each workgroup then
// stages half of the activation operand): adds the S partial results in split order, then does what EpiQKV does: rotates
// Q and K, stores Q as a pair of planes (hi, lo) and K and V into their cache slots.  `part` is [S][M][ncols] fp32 in the
// packed column order of the fused matrix (a band = eight channels of a head and, eight columns further on, their rotary
// partners), already scaled by the rows' RMSNorm factors.
// grid = (Hq + 2*Hkv heads, groups of eight rows), 256 threads: a wave is 8 rows x 8 channel pairs (lane = row % 8 +
// 8 * pair), so that a store instruction covers runs of eight channels of a row (Q, K tiles) and of eight slots of a
// channel (V tiles); wave w takes pairs 8w .. 8w+7 of every 32.
struct QkvFinishArgs {
    static constexpr int MAX_SPLITS = 4;
    const float* part;
    int S;  // splits, at most MAX_SPLITS
    size_t split_stride;
    int ncols;
    int Hq, Hkv, D;
    u16* q_out;
    int ldq;
    size_t q_plane;
    u16* kc;
    u16* vc;
    int max_seq;
    const float* rope_cos;
    const float* rope_sin;
    RowPlan plan;
    const int32_t* dev_prefix_len;  // may be nullptr; a device prefix length other than plan.P: nothing goes to the cache
};

// All loads of a thread (its channel pairs x the splits, the rotary factors, the device prefix length) are requested
// before the first is used: the kernel is one memory round trip and its stores.
template <int D>
__global__ __launch_bounds__(256) void qkv_finish_kernel(QkvFinishArgs a) {
    constexpr int half = D / 2, bph = D / 16, IT = half / 32, MAXS = QkvFinishArgs::MAX_SPLITS;
    const int head = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = blockIdx.y * 8 + (lane & 7);
    if (m >= a.plan.M) return;
    const int32_t dev_P = a.dev_prefix_len ? *a.dev_prefix_len : a.plan.P;
    const float* row = a.part + (size_t)m * a.ncols;
    const bool rotate = head < a.Hq + a.Hkv;
    float p_lo[IT][MAXS], p_hi[IT][MAXS], cs[IT], sn[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int dd = it * 32 + wave * 8 + (lane >> 3);
        const int n_lo = (head * bph + (dd >> 3)) * 16 + (dd & 7);  // channel dd; its partner dd + D/2 sits 8 columns on
#pragma unroll
        for (int sp = 0; sp < MAXS; ++sp) {  // a split that is not there: split 0 again, not added
            const float* ps = row + (sp < a.S ? (size_t)sp * a.split_stride : 0);
            p_lo[it][sp] = ps[n_lo];
            p_hi[it][sp] = ps[n_lo + 8];
        }
        cs[it] = rotate ? a.rope_cos[m * half + dd] : 1.f;
        sn[it] = rotate ? a.rope_sin[m * half + dd] : 0.f;
    }
    const bool cache_ok = dev_P == a.plan.P;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int dd = it * 32 + wave * 8 + (lane >> 3);
        float x_lo = 0.f, x_hi = 0.f;
#pragma unroll
        for (int sp = 0; sp < MAXS; ++sp) {
            if (sp < a.S) {
                x_lo += p_lo[it][sp];
                x_hi += p_hi[it][sp];
            }
        }
        if (rotate) {
            const float r_lo = x_lo * cs[it] - x_hi * sn[it], r_hi = x_hi * cs[it] + x_lo * sn[it];
            if (head < a.Hq) {
                u16* q = a.q_out + (size_t)m * a.ldq + head * D;
                const u16 h_lo = f32_to_elem(r_lo), h_hi = f32_to_elem(r_hi);
                q[dd] = h_lo;
                q[half + dd] = h_hi;
                q[a.q_plane + dd] = f32_to_elem(r_lo - elem_to_f32(h_lo));
                q[a.q_plane + half + dd] = f32_to_elem(r_hi - elem_to_f32(h_hi));
            } else if (cache_ok) {
                u16* kp = a.kc + (size_t)(head - a.Hq) * a.max_seq * D;
                kp[k_cache_offset(D, a.plan.slot(m), dd)] = f32_to_elem(r_lo);
                kp[k_cache_offset(D, a.plan.slot(m), half + dd)] = f32_to_elem(r_hi);
            }
        } else if (cache_ok) {
            u16* vp = a.vc + (size_t)(head - a.Hq - a.Hkv) * a.max_seq * D;
            vp[v_cache_offset(D, a.plan.slot(m), dd)] = f32_to_elem(x_lo);
            vp[v_cache_offset(D, a.plan.slot(m), half + dd)] = f32_to_elem(x_hi);
        }
    }
}

// cos/sin of pos(m) * theta^(-2d/D), evaluated in double and rounded once to fp32.  As the first kernel of a
// pass it also clears the status word that the later kernels OR their flags into, and, for a pass that will be
// followed by sampling from cached root logits (root.logits != nullptr), its last ROOT_STATS_PARTS workgroups leave the
// softmax statistics of those logits, slice by slice (see SampleArgs in duo_sample.h): work that is off the
// critical path here and would otherwise need a launch of its own.
struct RootStatsArgs {
    const float* logits;  // fp32 [V], or nullptr: no statistics wanted
    int V;
    double T;
    double* out;  // [ROOT_STATS_PARTS][2]
};

__global__ __launch_bounds__(256) void rope_table_kernel(RowPlan plan, int D, double theta, float* __restrict__ rc,
                                                          float* __restrict__ rs, int32_t* status, RootStatsArgs root) {
    __shared__ double sm[16];
    const int m = blockIdx.x, half = D / 2;
    if (m == 0 && threadIdx.x == 0 && status) *status = 0;
    if (m >= plan.M) {  // statistics of one slice of the root logits
        if (!root.logits) return;
        const int sl = m - plan.M, len = (root.V + ROOT_STATS_PARTS - 1) / ROOT_STATS_PARTS;
        const int v0 = sl * len, v1 = min(root.V, v0 + len);
        double zmax, Z;
        slice_stats(root.logits, v0, v1, root.T, sm, zmax, Z);
        if (threadIdx.x == 0) {
            root.out[2 * sl] = zmax;
            root.out[2 * sl + 1] = Z;
        }
        return;
    }
    for (int d = threadIdx.x; d < half; d += blockDim.x) {
        const double ang = (double)plan.pos(m) * pow(theta, -2.0 * (double)d / (double)D);
        rc[m * half + d] = (float)cos(ang);
        rs[m * half + d] = (float)sin(ang);
    }
}

// The device-side input check of a call that scores no row: the status word starts clean unless the device's prefix
// length is not the host's.
__global__ void status_init_kernel(int32_t* status, const int32_t* prefix_len, int host_P) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *status = (prefix_len && *prefix_len != host_P) ? 2 : 0;
}

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Row m of a paired operand buffer (hi at row m, lo at row pair_rows + m; `tiles` row tiles per K step) as an operand
// of its own for a one-row product: one tile per K step, hi in row 0, lo in row 8, all other rows zero.
// grid = K/32 workgroups of one wave.
__global__ __launch_bounds__(64) void last_row_operand_kernel(const u16* __restrict__ src, int m, int pair_rows, int tiles,
                                                              u16* __restrict__ dst) {
    const int ks = blockIdx.x, lane = threadIdx.x, r = lane & 15, g = lane >> 4;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (r == 0 || r == 8) {
        const int row = r == 0 ? m : pair_rows + m;
        v = *reinterpret_cast<const u32x4*>(src + (((size_t)ks * tiles + (row >> 4)) * 64 + g * 16 + (row & 15)) * 8);
    }
    *reinterpret_cast<u32x4*>(dst + ((size_t)ks * 64 + lane) * 8) = v;
}

// Plain streaming read of `chunks` 16-byte chunks (the ceiling a weight stream can reach on the device): every lane
// keeps eight independent 16-byte loads in flight, 1 KiB per wave and load instruction as in the projection kernels,
// with ordinary loads or (NT) with the non-temporal hint the projection kernels give their weight loads;
// the xor of everything read goes to sink[workgroup] so that the loads cannot be dropped.
template <bool NT>
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t chunks, uint32_t* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 7 * stride < chunks; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = NT ? __builtin_nontemporal_load(src + i + j * stride) : src[i + j * stride];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j];
    }
    for (; i < chunks; i += stride) acc ^= src[i];
    uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o, 64);
    if ((threadIdx.x & 63) == 0) atomicXor(sink + blockIdx.x, x);
}
