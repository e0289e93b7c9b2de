// Skinny weight-streaming products y = x W^T for M <= 80 rows (the projections of the target
// pass, Alg. 1 right column).  The weights are read exactly once from HBM, straight into MFMA
// operand registers; the few activation rows are re-read from L2 by every workgroup.
//
// Work split: a workgroup owns NT tiles of 16 weight rows and the whole K range; its NW waves
// take the 32-wide K steps round-robin (so at any moment the workgroup reads NW*64 contiguous
// bytes of each row), keep PF steps of loads in flight, and their partial sums are added in
// wave order through LDS (deterministic, no float atomics).  The epilogue functor decides which
// weight rows form a tile and what happens to the sums (plain store, residual add, SwiGLU,
// rotary embedding + KV-cache scatter).
//
// Activation precision: an activation a is carried as a bf16 pair (hi, lo) with hi = bf16(a),
// lo = bf16(a - hi), i.e. 16 mantissa bits.  The pair occupies two ROWS of the MFMA A operand:
// row m holds hi, row m + pair_rows holds lo, and the epilogue adds the two output rows.  For the
// common M <= 8 case both halves fit the one 16-row tile an MFMA needs anyway, so the extra
// precision costs nothing; a single bf16 per activation would leave rounding noise of ~0.1 in the
// logits of a 32-layer model.
#pragma once
#include "duo_common.h"

template <int MT, int NT, int NW, int PF, class Epi>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_kernel(const u16* __restrict__ X, int ldx, int K, int quads,
                                                               int pair_quads, Epi epi) {
    __shared__ f32x4 red[NW * MT * NT * 64];
    const int tile = blockIdx.x;
    // the wave index must live in a scalar register: MFMA ignores the EXEC mask, so every branch
    // around an MFMA has to be a scalar (wave-uniform) branch, never lane predication
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;

    const u16* wp[NT];
    const u16* xp[MT];
#pragma unroll
    for (int t = 0; t < NT; ++t) wp[t] = epi.row_ptr(tile, t, c) + g * 8;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) xp[mt] = X + (size_t)(mt * 16 + c) * ldx + g * 8;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int steps = K >> 5;
    const int ni = (steps - wave + NW - 1) / NW;  // this wave's steps: wave, wave + NW, ...
    if (ni > 0) {
        bf16x8 bb[PF][NT], aa[PF][MT];
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int i = p < ni ? p : ni - 1;
            const int off = (wave + NW * i) << 5;
#pragma unroll
            for (int t = 0; t < NT; ++t) bb[p][t] = load_frag_stream(wp[t] + off);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) aa[p][mt] = load_frag(xp[mt] + off);
        }
        for (int i0 = 0; i0 < ni; i0 += PF) {
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                const int i = i0 + p;
                bf16x8 b[NT], a[MT];
#pragma unroll
                for (int t = 0; t < NT; ++t) b[t] = bb[p][t];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) a[mt] = aa[p][mt];
                int in = i + PF;
                in = in < ni ? in : ni - 1;  // tail: re-read the last step (in bounds, L1 hit)
                const int off = (wave + NW * in) << 5;
#pragma unroll
                for (int t = 0; t < NT; ++t) bb[p][t] = load_frag_stream(wp[t] + off);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) aa[p][mt] = load_frag(xp[mt] + off);
                if (i < ni) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int t = 0; t < NT; ++t) acc[mt][t] = mfma16(a[mt], b[t], acc[mt][t]);
                }
            }
        }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t) red[((wave * MT + mt) * NT + t) * 64 + lane] = acc[mt][t];
    __syncthreads();
    // output quad qi = rows 4qi .. 4qi+3, column c; its hi sums sit in MFMA tile qi/4, lane group
    // qi%4, its lo sums pair_quads quads further on (pair_quads == 0: rows are not paired)
    for (int idx = threadIdx.x; idx < quads * 16; idx += NW * 64) {
        const int qi = idx >> 4, c = idx & 15;
        const int slot_hi = (qi >> 2) * NT * 64 + (qi & 3) * 16 + c;
        const int ql = qi + pair_quads;
        const int slot_lo = (ql >> 2) * NT * 64 + (ql & 3) * 16 + c;
        f32x4 v[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            f32x4 s = red[slot_hi + t * 64];
#pragma unroll
            for (int w = 1; w < NW; ++w) s += red[w * MT * NT * 64 + slot_hi + t * 64];
            if (pair_quads) {
                f32x4 l = red[slot_lo + t * 64];
#pragma unroll
                for (int w = 1; w < NW; ++w) l += red[w * MT * NT * 64 + slot_lo + t * 64];
                s += l;
            }
            v[t] = s;
        }
        epi.store(tile, qi, c, v);
    }
}

// ---- epilogues -------------------------------------------------------------------------------
// store(tile, qi, c, v): v[t][i] is the sum for row m = 4*qi + i, column c of tile slot t.

struct EpiStoreF32 {  // y[m][n] = sum ; tile slot t covers rows (tile*NT + t)*16 .. +16 of W
    const u16* W;
    int ldw, N, M, NT;
    float* Y;
    int ldy;
    __device__ __forceinline__ const u16* row_ptr(int tile, int t, int c) const {
        int n = (tile * NT + t) * 16 + c;
        n = n < N ? n : N - 1;
        return W + (size_t)n * ldw;
    }
    template <int NTT>
    __device__ __forceinline__ void store(int tile, int qi, int c, const f32x4 (&v)[NTT]) const {
#pragma unroll
        for (int t = 0; t < NTT; ++t) {
            const int n = (tile * NT + t) * 16 + c;
            if (n >= N) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = qi * 4 + i;
                if (m < M) Y[(size_t)m * ldy + n] = v[t][i];
            }
        }
    }
};

struct EpiResidual {  // x[m][n] += sum  (fp32 residual stream, each element owned by one workgroup)
    const u16* W;
    int ldw, N, M, NT;
    float* X;
    int ldx;
    __device__ __forceinline__ const u16* row_ptr(int tile, int t, int c) const {
        int n = (tile * NT + t) * 16 + c;
        n = n < N ? n : N - 1;
        return W + (size_t)n * ldw;
    }
    template <int NTT>
    __device__ __forceinline__ void store(int tile, int qi, int c, const f32x4 (&v)[NTT]) const {
#pragma unroll
        for (int t = 0; t < NTT; ++t) {
            const int n = (tile * NT + t) * 16 + c;
            if (n >= N) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = qi * 4 + i;
                if (m < M) X[(size_t)m * ldx + n] += v[t][i];
            }
        }
    }
};

struct EpiSwiGLU {  // slot 0 = gate row n, slot 1 = up row n; act[m][n] = silu(gate) * up as a bf16 pair
    const u16* Wg;
    const u16* Wu;
    int ldw, F, M;
    u16* act;  // [2 * pair_rows ..][ld]: row m hi, row pair_rows + m lo
    int ld, pair_rows;
    __device__ __forceinline__ const u16* row_ptr(int tile, int t, int c) const {
        int n = tile * 16 + c;
        n = n < F ? n : F - 1;
        return (t == 0 ? Wg : Wu) + (size_t)n * ldw;
    }
    __device__ __forceinline__ void store(int tile, int qi, int c, const f32x4 (&v)[2]) const {
        const int n = tile * 16 + c;
        if (n >= F) return;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = qi * 4 + i;
            if (m < M) {
                const float gate = v[0][i], up = v[1][i];
                const float a = gate / (1.f + expf(-gate)) * up;
                const u16 hi = f32_to_bf16(a);
                act[(size_t)m * ld + n] = hi;
                act[(size_t)(pair_rows + m) * ld + n] = f32_to_bf16(a - bf16_to_f32(hi));
            }
        }
    }
};

// Fused Q/K/V projection: a tile pairs rows d and d + D/2 of one head (slot 0 / slot 1), the two
// halves of a rotary pair, so the rotation is thread-local.  Q goes to the query buffer as a bf16 pair
// (hi plane, lo plane), K
// (rotated) and V into their cache slots; V is stored transposed [head][d][slot].
struct EpiQKV {
    const u16* Wq;
    const u16* Wk;
    const u16* Wv;
    int ldw, Hq, Hkv, D, half, bph;  // bph = (D/2)/16 tiles per head
    u16* q_out;  // hi plane; the lo plane starts q_plane elements further on
    int ldq;
    size_t q_plane;
    u16* kc;  // this layer: [Hkv][max_seq][D]
    u16* vc;  // this layer: [Hkv][D][max_seq]
    int max_seq;
    const float* rope_cos;  // [rows][D/2]
    const float* rope_sin;
    RowPlan plan;
    __device__ __forceinline__ const u16* row_ptr(int tile, int t, int c) const {
        int head = tile / bph;
        const int blk = tile - head * bph;
        const int r = t * half + blk * 16 + c;
        if (head < Hq) return Wq + (size_t)(head * D + r) * ldw;
        head -= Hq;
        if (head < Hkv) return Wk + (size_t)(head * D + r) * ldw;
        head -= Hkv;
        return Wv + (size_t)(head * D + r) * ldw;
    }
    __device__ __forceinline__ void store(int tile, int qi, int c, const f32x4 (&v)[2]) const {
        int head = tile / bph;
        const int d = (tile - head * bph) * 16 + c;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = qi * 4 + i;
            if (m >= plan.M) continue;
            const float lo = v[0][i], hi = v[1][i];
            if (head < Hq + Hkv) {
                const float cs = rope_cos[m * half + d], sn = rope_sin[m * half + d];
                const float rl = lo * cs - hi * sn, rh = hi * cs + lo * sn;
                if (head < Hq) {
                    u16* q = q_out + (size_t)m * ldq + head * D + d;
                    const u16 l1 = f32_to_bf16(rl), h1 = f32_to_bf16(rh);
                    q[0] = l1;
                    q[half] = h1;
                    q[q_plane] = f32_to_bf16(rl - bf16_to_f32(l1));
                    q[q_plane + half] = f32_to_bf16(rh - bf16_to_f32(h1));
                } else {
                    u16* kp = kc + ((size_t)(head - Hq) * max_seq + plan.slot(m)) * D + d;
                    kp[0] = f32_to_bf16(rl);
                    kp[half] = f32_to_bf16(rh);
                }
            } else {
                u16* vp = vc + ((size_t)(head - Hq - Hkv) * D + d) * max_seq + plan.slot(m);
                vp[0] = f32_to_bf16(lo);
                vp[(size_t)half * max_seq] = f32_to_bf16(hi);
            }
        }
    }
};

// rows: output rows M; paired: activations are bf16 pairs (rows m and pair_rows + m of X).
template <int MT, int NT, class Epi>
static inline void launch_gemm(const u16* X, int ldx, int K, int tiles, int quads, int pair_quads, const Epi& epi,
                               hipStream_t s) {
    constexpr int NW = MT <= 2 ? 8 : (MT <= 6 ? 4 : 2);  // keeps the reduction buffer within 64 KB of LDS
    constexpr int PF = MT <= 2 ? 8 : (MT <= 4 ? 4 : 2);
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, NT, NW, PF, Epi>), dim3(tiles), dim3(NW * 64), 0, s, X, ldx, K, quads,
                       pair_quads, epi);
}

// Rows of the A operand for M paired activations: hi rows [0, pair_rows), lo rows [pair_rows, 2*pair_rows).
static inline int pair_rows_for(int M) { return (M + 7) / 8 * 8; }
static inline int a_tiles_for(int M, bool paired) { return paired ? (2 * pair_rows_for(M) + 15) / 16 : (M + 15) / 16; }

template <int NT, class Epi>
static inline void launch_gemm_rows(int M, bool paired, const u16* X, int ldx, int K, int tiles, const Epi& epi,
                                    hipStream_t s) {
    const int mt = a_tiles_for(M, paired);
    const int quads = paired ? pair_rows_for(M) / 4 : (M + 3) / 4;
    const int pq = paired ? pair_rows_for(M) / 4 : 0;
    switch (mt) {
        case 1: launch_gemm<1, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
        case 2: launch_gemm<2, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
        case 3: launch_gemm<3, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
        case 4: launch_gemm<4, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
        case 5: launch_gemm<5, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
        case 6: launch_gemm<6, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
        case 7: launch_gemm<7, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
        case 8: launch_gemm<8, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
        case 9: launch_gemm<9, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
        default: launch_gemm<10, NT>(X, ldx, K, tiles, quads, pq, epi, s); break;
    }
}
