// Masked attention of the verify pass: every row attends to the shared prefix, the optional root
// token and the earlier tokens of its own draft sequence (independent sequences, Sec. 3.2).
//
// The prefix keys/values of one KV head are read ONCE for all rows and all query heads of the
// group: a workgroup takes one (kv head, key chunk), each of its four waves a share of the
// chunk's 32-key blocks.  Per block a wave computes S^T = K Q^T and O^T += V^T P^T with MFMA:
//   - K rows and V^T rows (values are cached transposed) are loaded straight from HBM in MFMA
//     operand layout, 16 bytes per lane, no LDS staging -- each byte is consumed by one wave;
//   - the key permutation inside a block is chosen so that the S^T accumulator of a lane
//     already holds the eight consecutive keys its P^T operand needs: no cross-lane traffic
//     between the two products;
//   - queries and softmax weights enter the MFMAs as bf16 pairs (hi + lo), keys and values are the
//     cache's bf16;
//   - the softmax is online (running max / sum per row), reduced across the four lane groups
//     with wavefront shuffles.
// The four waves are merged through LDS in a fixed chain, chunk partials (max, sum,
// unnormalised O) go to scratch and a small kernel merges the chunks in chunk order.
#pragma once
#include "duo_common.h"
#include "duo_gemm.h"

struct AttnArgs {
    const u16* q;  // queries as bf16 pairs: hi plane [rows][Hq*D], lo plane q_plane elements further on
    int ldq;
    size_t q_plane;
    const u16* kc;  // this layer: [Hkv][max_seq][D]
    const u16* vc;  // this layer: [Hkv][D][max_seq]
    int max_seq, group;
    RowPlan plan;
    int Ktot;             // P + M keys in play
    int blocks_per_wave;  // 32-key blocks per wave; a chunk is 4 * blocks_per_wave blocks
    int nchunks;
    int mq_pad;           // padded number of (row, query-head-in-group) pairs
    float scale_log2;     // log2(e) / sqrt(D)
    float* part;          // [Hkv][mq_pad][nchunks][D + 4]: O (unnormalised), max, sum
};

template <int D, int MTW>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnArgs a) {
    constexpr int KS = D / 32;  // MFMA K steps of the QK^T product
    constexpr int DT = D / 16;  // 16-channel tiles of the PV product
    __shared__ f32x4 lds_o[MTW * DT * 64];
    __shared__ float lds_ml[MTW][2][16];

    const int cb = blockIdx.x, hk = blockIdx.y, mg = blockIdx.z;
    // scalar wave index: MFMA ignores the EXEC mask, so all control flow around it must be wave-uniform
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;
    const int MQ = a.plan.M * a.group;

    // query operand (B of S^T = K Q^T): column c of tile mt is pair r = (row m, head gq of the group)
    // Visibility of draft slots, branch-free: with mk = key - P, row m sees mk < R (prefix and root)
    // and vis_lo <= mk <= vis_hi (its own sequence up to itself).
    bf16x8 qf[MTW][KS], ql[MTW][KS];
    int vis_lo[MTW], vis_hi[MTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const int r = (mg * MTW + mt) * 16 + c;
        const bool ok = r < MQ;
        const int m = ok ? r / a.group : 0, gq = ok ? r % a.group : 0;
        const int R = a.plan.R;
        vis_lo[mt] = !ok ? 0x7fffffff : (m < R ? 0 : R + ((m - R) / a.plan.k) * a.plan.k);
        vis_hi[mt] = ok ? m : -1;
        const u16* qp = a.q + (size_t)m * a.ldq + (hk * a.group + gq) * D + g * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            Frag8 f;
            f.q = ok ? *reinterpret_cast<const u32x4*>(qp + ks * 32) : u32x4{0u, 0u, 0u, 0u};
            qf[mt][ks] = f.v;
            f.q = ok ? *reinterpret_cast<const u32x4*>(qp + a.q_plane + ks * 32) : u32x4{0u, 0u, 0u, 0u};
            ql[mt][ks] = f.v;
        }
    }

    f32x4 o[MTW][DT];
    float m_run[MTW], l_run[MTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        m_run[mt] = -INFINITY;
        l_run[mt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[mt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const u16* kbase = a.kc + (size_t)hk * a.max_seq * D + g * 8;
    const u16* vbase = a.vc + ((size_t)hk * D + c) * a.max_seq + g * 8;
    const int b0 = (cb * 4 + wave) * a.blocks_per_wave;
    for (int ib = 0; ib < a.blocks_per_wave; ++ib) {
        const int kb = (b0 + ib) * 32;
        if (kb >= a.Ktot) break;  // wave-uniform
        // ---- S^T tiles: tile t, MFMA row r' = 4*g' + i' is key kb + 8*g' + 4*t + i'
        f32x4 s[2][MTW];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            int key = kb + (c >> 2) * 8 + t * 4 + (c & 3);
            key = key < a.Ktot ? key : a.Ktot - 1;
            const u16* kp = kbase + (size_t)key * D;
            bf16x8 kf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[ks] = load_frag_stream(kp + ks * 32);
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16(kf[ks], ql[mt][ks], acc);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16(kf[ks], qf[mt][ks], acc);
                s[t][mt] = acc;
            }
        }
        // ---- V^T operands: lane (channel dt*16 + c, keys kb + 8g .. +8)
        bf16x8 vf[DT];
        const bool tail = kb + 32 > a.Ktot;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            Frag8 f;
            f.q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vbase + (size_t)dt * 16 * a.max_seq + kb));
            if (tail) {  // slots at or beyond Ktot may hold anything: zero them (0 * NaN would poison O)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (kb + g * 8 + j >= a.Ktot) f.h[j] = 0;
            }
            vf[dt] = f.v;
        }
        // ---- mask, online softmax, P^T operand
        const bool masked = kb + 32 > a.plan.P;  // block touches draft slots or the end
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
            float sc[8];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) sc[t * 4 + i] = s[t][mt][i] * a.scale_log2;
            if (masked) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int mk = kb + g * 8 + j - a.plan.P;
                    const bool vis = (mk < a.plan.R) | ((mk >= vis_lo[mt]) & (mk <= vis_hi[mt]));
                    sc[j] = vis ? sc[j] : -INFINITY;
                }
            }
            float bm = sc[0];
#pragma unroll
            for (int j = 1; j < 8; ++j) bm = fmaxf(bm, sc[j]);
            bm = fmaxf(bm, __shfl_xor(bm, 16, 64));
            bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
            const float m_new = fmaxf(m_run[mt], bm);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = exp2f(m_run[mt] - m_safe);
            m_run[mt] = m_new;
            // the weights enter the MFMA as a bf16 pair hi + lo (16 mantissa bits): rounding them to a
            // single bf16 would add as much noise to O as the bf16 rounding of O itself
            Frag8 pf, pl;
            float ps = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float p = exp2f(sc[j] - m_safe);
                const u16 hi = f32_to_bf16(p);
                pf.h[j] = hi;
                pl.h[j] = f32_to_bf16(p - bf16_to_f32(hi));
                ps += p;
            }
            l_run[mt] = l_run[mt] * alpha + ps;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                f32x4 acc = o[mt][dt] * alpha;
                acc = mfma16(vf[dt], pl.v, acc);
                o[mt][dt] = mfma16(vf[dt], pf.v, acc);
            }
        }
    }
    // lane-group partial sums -> row sums (max is already uniform across lane groups)
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        l_run[mt] += __shfl_xor(l_run[mt], 16, 64);
        l_run[mt] += __shfl_xor(l_run[mt], 32, 64);
    }

    // ---- merge the four waves in a fixed chain: 2 <- 3, 1 <- 2, 0 <- 1 (one LDS buffer)
    for (int sender = 3; sender >= 1; --sender) {
        if (wave == sender) {
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) lds_o[(mt * DT + dt) * 64 + lane] = o[mt][dt];
                if (g == 0) {
                    lds_ml[mt][0][c] = m_run[mt];
                    lds_ml[mt][1][c] = l_run[mt];
                }
            }
        }
        __syncthreads();
        if (wave == sender - 1) {
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) {
                const float mo = lds_ml[mt][0][c], lo = lds_ml[mt][1][c];
                const float mn = fmaxf(m_run[mt], mo);
                const float ms = mn == -INFINITY ? 0.f : mn;
                const float sa = exp2f(m_run[mt] - ms), sb = exp2f(mo - ms);
                m_run[mt] = mn;
                l_run[mt] = l_run[mt] * sa + lo * sb;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
                    o[mt][dt] = o[mt][dt] * sa + lds_o[(mt * DT + dt) * 64 + lane] * sb;
            }
        }
        __syncthreads();
    }
    if (wave == 0) {
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
            const int r = (mg * MTW + mt) * 16 + c;
            if (r >= MQ) continue;
            float* pp = a.part + (((size_t)hk * a.mq_pad + r) * a.nchunks + cb) * (D + 4);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                *reinterpret_cast<f32x4*>(pp + dt * 16 + g * 4) = o[mt][dt];  // O^T rows 4g..4g+3 of tile dt
            if (g == 0) {
                pp[D] = m_run[mt];
                pp[D + 1] = l_run[mt];
            }
        }
    }
}

// Merge the chunk partials of one (row, query head) in chunk order, normalise, store as a bf16 pair
// into the O projection's operand buffer (tile order; hi = operand row m, lo = row m + pair_rows).
template <int D>
__global__ __launch_bounds__(64) void attn_combine_kernel(const float* __restrict__ part, int nchunks, int mq_pad, int group,
                                                           int M, u16* __restrict__ out, int tiles, int pair_rows) {
    const int r = blockIdx.x, hk = blockIdx.y;
    const int m = r / group, gq = r % group;
    if (m >= M) return;
    const float* pp = part + ((size_t)hk * mq_pad + r) * nchunks * (D + 4);
    float mx = -INFINITY;
    for (int cb = 0; cb < nchunks; ++cb) mx = fmaxf(mx, pp[(size_t)cb * (D + 4) + D]);
    float L = 0.f;
    float acc[D / 64];
#pragma unroll
    for (int e = 0; e < D / 64; ++e) acc[e] = 0.f;
    for (int cb = 0; cb < nchunks; ++cb) {
        const float* p = pp + (size_t)cb * (D + 4);
        const float mc = p[D];
        if (mc == -INFINITY) continue;
        const float w = exp2f(mc - mx);
        L += p[D + 1] * w;
#pragma unroll
        for (int e = 0; e < D / 64; ++e) acc[e] += p[threadIdx.x + e * 64] * w;
    }
    const int col0 = (hk * group + gq) * D;
#pragma unroll
    for (int e = 0; e < D / 64; ++e) {
        const float o = acc[e] / L;
        const u16 hi = f32_to_bf16(o);
        const int col = col0 + threadIdx.x + e * 64;
        out[operand_offset(m, col, tiles)] = hi;
        out[operand_offset(pair_rows + m, col, tiles)] = f32_to_bf16(o - bf16_to_f32(hi));
    }
}
