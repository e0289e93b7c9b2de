// Projections over many rows (prefill chunks of 81..1024 prompt tokens; the target model's share of the
// time to first token, Sec. 4.1).  With that many rows the product is no longer a weight stream with a
// few activation rows beside it: both operands are re-used and both are staged in LDS.
//
// A workgroup owns a block of 2*WM row tiles (16 rows each) x 2*WN weight bands (16 columns each); its four
// consumer waves form a 2 x 2 grid, each with WM x WN accumulator tiles.  Both operands already lie in
// MFMA-tile order in global memory (duo_gemm.h), so a stage is a list of 1 KiB tiles: per K step the block's
// hi tiles, its lo tiles (the activations are bf16 pairs, hi and lo products add into the same accumulators)
// and its weight tiles.  A fifth wave does nothing but move tiles: 16-byte global -> LDS loads into a
// three-deep ring of stages, two stages ahead, handed over with one barrier per stage (bare s_barrier
// behind a counted wait in the producer, exactly as in gemm_wide_kernel).  The consumers touch no global
// memory inside the loop.
//
// Per K step a wave reads (2*WM + WN) KiB from LDS for 2*WM*WN MFMAs: 12 KiB per 32 MFMAs (512 cycles) at
// WM = WN = 4, i.e. 96 B/clk per compute unit, inside what LDS delivers; the block pulls (4*WM + 2*WN) KiB
// per K step through L2.
//
// Grid: x = blocks of bands, y = K splits (partial results, see EpiStoreF32), z = blocks of rows.
// ENT = bands per epilogue tile (2 for the rotary and SwiGLU epilogues, 1 otherwise).
#pragma once
#include "duo_gemm.h"

template <int WM, int WN, int KS, int ENT, class Epi>
__global__ __launch_bounds__(320) void gemm_block_kernel(const u16* __restrict__ X, const u16* __restrict__ W, int K,
                                                         int split_steps, int band_base, int nbands, int mh_total, int quads, RowScale rsc,
                                                         Epi epi) {
    constexpr int BMT = 2 * WM, BNT = 2 * WN;  // row tiles (hi) and bands per workgroup
    constexpr int PER = 2 * BMT + BNT;         // tiles per K step
    constexpr int ST = KS * PER;               // tiles per stage
    constexpr int NBUF = 3;
    static_assert(ST <= 63, "a stage's loads fit the memory counter");
    static_assert(WN % ENT == 0, "whole epilogue tiles per wave");
    __shared__ u32x4 lds[NBUF * ST * 64];
    __shared__ float row_scale[BMT * 16];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;  // scalar: MFMA ignores EXEC
    const int steps = K >> 5;
    const int k0 = blockIdx.y * split_steps;
    const int ns = min(steps - k0, split_steps);  // K steps of this split (the host makes it positive)
    const int rounds = (ns + KS - 1) / KS;
    const int row_tile0 = blockIdx.z * BMT, band0 = band_base + blockIdx.x * BNT;  // bands [band_base, nbands) are this launch's
    const int row0 = row_tile0 * 16, nrows = quads * 4;

    // RMSNorm factors of this block's rows (all five waves)
    if (rsc.full) {
        for (int i = threadIdx.x; i < BMT * 16; i += 320) {
            const int m = row0 + i;
            row_scale[i] = m < nrows ? 1.0f / sqrtf(rsc.full_row(m) * rsc.inv_d + rsc.eps) : 0.f;
        }
    } else if (rsc.part) {
        f32x4 rsv[RowScale::MAXQ];
        const int rend = min(row0 + BMT * 16, nrows);
        for (int r0 = row0 + wave * 8; r0 < rend; r0 += 5 * 8) {
            rsc.load(rsv, r0, nrows, lane);
            rsc.reduce(rsv, row_scale - row0, r0, nrows, lane);
        }
    }

    if (wave == 4) {
        // ---- producer: stage r goes to ring buffer r % 3; steps past the end re-read the last step
        const u32x4* xg = reinterpret_cast<const u32x4*>(X) + lane;
        const u32x4* wg = reinterpret_cast<const u32x4*>(W) + lane;
        const int mt_total = 2 * mh_total;
        auto issue = [&](int r) {
            const int b = r % NBUF;
#pragma unroll
            for (int i = 0; i < ST; ++i) {
                const int ks = i / PER, t = i % PER;
                int st = r * KS + ks;
                st = k0 + (st < ns ? st : ns - 1);
                const u32x4* src;
                if (t < 2 * BMT) {  // hi tiles, then lo tiles; row tiles past the operand re-read its last one
                    int rt = row_tile0 + t % BMT;
                    rt = rt < mh_total ? rt : mh_total - 1;
                    src = xg + ((size_t)st * mt_total + (t / BMT) * mh_total + rt) * 64;
                } else {  // bands past the matrix re-read its last one
                    int bd = band0 + (t - 2 * BMT);
                    bd = bd < nbands ? bd : nbands - 1;
                    src = wg + ((size_t)bd * steps + st) * 64;
                }
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                                 (__attribute__((address_space(3))) void*)(lds + (b * ST + i) * 64), 16, 0, 0);
            }
        };
        // vmcnt(ST): everything but the youngest stage has landed (expcnt and lgkmcnt fields left at their maxima)
        constexpr int WAIT_ALL_BUT_ONE_STAGE = (ST & 15) | ((ST >> 4) << 14) | (7 << 4) | (15 << 8);
        issue(0);
        issue(1);
        __builtin_amdgcn_s_waitcnt(WAIT_ALL_BUT_ONE_STAGE & ~(15 << 8));  // and lgkmcnt(0): this wave's row scales are written
        __builtin_amdgcn_s_barrier();
        for (int r = 0; r < rounds; ++r) {
            issue(r + 2);  // its buffer was drained in round r - 1
            __builtin_amdgcn_s_waitcnt(WAIT_ALL_BUT_ONE_STAGE);  // stage r + 1 has landed
            __builtin_amdgcn_s_barrier();
        }
        __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));  // vmcnt(0): nothing is in flight towards LDS when this wave ends
        return;
    }

    // ---- consumers: wave (wm, wn) of the 2 x 2 grid
    epi.arm();
    const int wm = wave >> 1, wn = wave & 1;
    f32x4 acc[WM][WN];
#pragma unroll
    for (int m = 0; m < WM; ++m)
#pragma unroll
        for (int t = 0; t < WN; ++t) acc[m][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    __syncthreads();  // stage 0 is in LDS, the row scales are written
    for (int r = 0; r < rounds; ++r) {
        const u32x4* stage = lds + (r % NBUF) * ST * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (r * KS + ks < ns) {  // wave-uniform
                const u32x4* st = stage + ks * PER * 64;
                elem8 ah[WM], al[WM], b[WN];
#pragma unroll
                for (int m = 0; m < WM; ++m) {
                    Frag8 f, g;
                    f.q = st[(wm * WM + m) * 64];
                    g.q = st[(BMT + wm * WM + m) * 64];
                    ah[m] = f.v;
                    al[m] = g.v;
                }
#pragma unroll
                for (int t = 0; t < WN; ++t) {
                    Frag8 f;
                    f.q = st[(2 * BMT + wn * WN + t) * 64];
                    b[t] = f.v;
                }
#pragma unroll
                for (int m = 0; m < WM; ++m)
#pragma unroll
                    for (int t = 0; t < WN; ++t) acc[m][t] = mfma16(b[t], ah[m], acc[m][t]);
#pragma unroll
                for (int m = 0; m < WM; ++m)
#pragma unroll
                    for (int t = 0; t < WN; ++t) acc[m][t] = mfma16(b[t], al[m], acc[m][t]);
            }
        }
        __syncthreads();  // stage r + 1 is in LDS; stage r's buffer may be refilled
    }

    // The weights are the FIRST operand of the products above, so a lane's accumulator quad is one output row
    // (lane % 16 of the row tile) and four consecutive columns (4 * (lane / 16) .. +3 of the band): vector stores.
#pragma unroll
    for (int m = 0; m < WM; ++m) {
        const int row = (row_tile0 + wm * WM + m) * 16 + (lane & 15);
        const float rs = (rsc.part && row < nrows) ? row_scale[row - row0] : 1.f;
#pragma unroll
        for (int t = 0; t < WN; t += ENT) {
            const int band = band0 + wn * WN + t;
            if (band >= nbands) continue;  // wave-uniform
            f32x4 v[ENT];
#pragma unroll
            for (int e = 0; e < ENT; ++e) v[e] = acc[m][t + e] * rs;
            epi.store4(band / ENT, row, 4 * (lane >> 4), v);
        }
    }
}

// Launch for M rows (operand of 2 * mh_total row tiles: hi tiles, then lo tiles) over the bands [band_begin, band_end) of
// 16 columns each, K split `splits` ways over the grid's y dimension (returns the number of splits actually used).
template <int WM, int WN, int ENT, class Epi>
static inline int launch_block_range(const u16* X, const u16* W, int K, int band_begin, int band_end, int M, int splits,
                                     const RowScale& rsc, const Epi& epi, hipStream_t s) {
    constexpr int KS = (2 * (4 * WM + 2 * WN) <= 48) ? 2 : 1;  // stage of at most 48 KiB
    const int mh_total = pair_rows_for(M) / 16, quads = pair_rows_for(M) / 4;
    const int steps = K >> 5;
    int split_steps = (steps + splits - 1) / splits;
    split_steps = (split_steps + KS - 1) / KS * KS;
    const int S = (steps + split_steps - 1) / split_steps;
    const dim3 grid((band_end - band_begin + 2 * WN - 1) / (2 * WN), S, (mh_total + 2 * WM - 1) / (2 * WM));
    DUO_KERNEL_NAME("gemm_block_kernel<%d, %d, %d, %d, %s>", WM, WN, KS, ENT, Epi::NAME);
    DUO_LAUNCH((gemm_block_kernel<WM, WN, KS, ENT, Epi>), grid, dim3(320), s, X, W, K, split_steps, band_begin, band_end, mh_total,
               quads, rsc, epi);
    return S;
}
template <int WM, int WN, int ENT, class Epi>
static inline int launch_block(const u16* X, const u16* W, int K, int nbands, int M, int splits, const RowScale& rsc,
                               const Epi& epi, hipStream_t s) {
    return launch_block_range<WM, WN, ENT>(X, W, K, 0, nbands, M, splits, rsc, epi, s);
}

// A projection whose epilogue finishes the rows (no K split), for M > 80 rows.  Workgroups of 64 x 128 wave tiles are the
// faster ones but come in few, large units: when their count leaves the last round of workgroups (one per compute unit)
// mostly empty, the bands of that round are given to workgroups of 64 x 64 wave tiles instead, in a second launch.
// Cost model in rounds of the large tile: a round of small tiles takes 0.55 of one.
// `before_launch` is called in front of every launch (the caller's per-kernel timer).
template <int ENT, class Epi, class Hook>
static inline void launch_block_rows(const u16* X, const u16* W, int K, int nbands, int M, const RowScale& rsc, const Epi& epi,
                                     hipStream_t s, Hook before_launch) {
    constexpr int CUS = 256;
    const int rb = (pair_rows_for(M) / 16 + 7) / 8;  // row blocks (128 rows)
    const int n_large = (nbands + 15) / 16, n_small = (nbands + 7) / 8;
    const auto rounds = [](int wgs) { return (wgs + CUS - 1) / CUS; };
    const float all_large = (float)rounds(n_large * rb), all_small = 0.55f * (float)rounds(n_small * rb);
    const int full = (n_large * rb) / CUS;                    // full rounds of large workgroups
    const int main_blocks = full * CUS / rb;                  // whole band blocks (256 columns) inside them
    const int rest_bands = nbands - main_blocks * 16;
    const float mixed = (full > 0 && rest_bands > 0) ? (float)rounds(main_blocks * rb) + 0.55f * (float)rounds((rest_bands + 7) / 8 * rb)
                                                      : 1e30f;
    before_launch();
    if (mixed < all_large && mixed < all_small) {
        launch_block_range<4, 8, ENT>(X, W, K, 0, main_blocks * 16, M, 1, rsc, epi, s);
        before_launch();
        launch_block_range<4, 4, ENT>(X, W, K, main_blocks * 16, nbands, M, 1, rsc, epi, s);
    } else if (all_large <= all_small && n_large * rb >= 160) {
        launch_block_range<4, 8, ENT>(X, W, K, 0, nbands, M, 1, rsc, epi, s);
    } else {
        launch_block_range<4, 4, ENT>(X, W, K, 0, nbands, M, 1, rsc, epi, s);
    }
}
