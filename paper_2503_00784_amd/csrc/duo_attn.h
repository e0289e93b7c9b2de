// Masked attention of the verify pass: every row attends to the shared prefix, the optional root
// token and the earlier tokens of its own draft sequence (independent sequences, Sec. 3.2).
//
// The prefix keys/values of one KV head are read ONCE for all rows and all query heads of the
// group: a workgroup takes one (kv head, key chunk), each of its waves a share of the
// chunk's 32-key blocks.  Per block a wave computes S^T = K Q^T and O^T += V^T P^T with MFMA:
//   - K rows and V^T rows (values are cached transposed) are loaded straight from HBM in MFMA
//     operand layout, 16 bytes per lane, no LDS staging -- each byte is consumed by one wave
//     (loads with the non-temporal hint: nothing of the prefix is read twice in a pass);
//   - the key permutation inside a block is chosen so that the S^T accumulator of a lane
//     already holds the eight consecutive keys its P^T operand needs: no cross-lane traffic
//     between the two products;
//   - queries and softmax weights enter the MFMAs as bf16 pairs (hi + lo), keys and values are the
//     cache's bf16;
//   - the softmax is online (running max / sum per row), reduced across the four lane groups
//     with wavefront shuffles.
// The waves are merged through LDS in a fixed chain, chunk partials (max, sum, unnormalised O)
// go to scratch and are merged in chunk order: by the same workgroup when a head is one chunk (short
// prefixes: one kernel per layer), by a small second kernel otherwise.
#pragma once
#include "duo_common.h"
#include "duo_gemm.h"

struct AttnArgs {
    const u16* q;  // queries as bf16 pairs: hi plane [rows][Hq*D], lo plane q_plane elements further on
    int ldq;
    size_t q_plane;
    const u16* kc;  // this layer: [Hkv] planes of max_seq * D elements, tiled (k_cache_offset)
    const u16* vc;  // this layer: [Hkv] planes of max_seq * D elements, tiled (v_cache_offset)
    int max_seq, group;
    RowPlan plan;
    int Ktot;             // P + M keys in play
    int blocks_per_wave;  // 32-key blocks per wave; a chunk is (waves per workgroup) * blocks_per_wave blocks
    int nchunks;
    int mq_pad;           // padded number of (row, query-head-in-group) pairs
    float scale_log2;     // log2(e) / sqrt(D)
    float* part;          // [Hkv][mq_pad][nchunks][D + 4]: O (unnormalised), max, sum
    u16* out;             // attention output, operand layout of the O projection (bf16 pairs)
    int out_tiles, pair_rows;
};

// Merge the chunk partials (at most 64) of one (row, query head), normalise, store as a bf16 pair
// (hi = operand row m, lo = operand row m + pair_rows).  Called by one wave.  Lane cb takes chunk cb's
// max and sum (one load each instead of a chain of them), the maximum and the weighted sum are formed by
// fixed butterflies; the outputs are then added in chunk order, lane handling D/64 channels; the first eight
// chunks' outputs are requested together with the statistics, further ones four at a time.
template <int D>
__device__ __forceinline__ void attn_merge_row(const AttnArgs& a, int hk, int r, int lane) {
    const int m = r / a.group, gq = r % a.group;
    const float* pp = a.part + ((size_t)hk * a.mq_pad + r) * a.nchunks * (D + 4);
    const bool has = lane < a.nchunks;
    const float mc = has ? pp[(size_t)lane * (D + 4) + D] : -INFINITY;
    const float lc = has ? pp[(size_t)lane * (D + 4) + D + 1] : 0.f;
    // the first eight chunks' outputs are requested with the statistics (they do not depend on them)
    constexpr int PRE = 8;
    float vp[PRE][D / 64];
#pragma unroll
    for (int i = 0; i < PRE; ++i) {
        const int cb = i < a.nchunks ? i : a.nchunks - 1;
#pragma unroll
        for (int e = 0; e < D / 64; ++e) vp[i][e] = pp[(size_t)cb * (D + 4) + lane + e * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
    float mx = mc;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    const float w = mc == -INFINITY ? 0.f : exp2f(mc - mx);  // this lane's chunk weight
    float L = lc * w;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) L += __shfl_xor(L, o, 64);
    float acc[D / 64];
#pragma unroll
    for (int e = 0; e < D / 64; ++e) acc[e] = 0.f;
#pragma unroll
    for (int i = 0; i < PRE; ++i) {
        const float wc = i < a.nchunks ? __shfl(w, i, 64) : 0.f;
#pragma unroll
        for (int e = 0; e < D / 64; ++e) acc[e] += vp[i][e] * wc;
    }
    for (int cb0 = PRE; cb0 < a.nchunks; cb0 += 4) {
        float v[4][D / 64], wc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int cb = cb0 + i < a.nchunks ? cb0 + i : a.nchunks - 1;
            wc[i] = cb0 + i < a.nchunks ? __shfl(w, cb, 64) : 0.f;
#pragma unroll
            for (int e = 0; e < D / 64; ++e) v[i][e] = pp[(size_t)cb * (D + 4) + lane + e * 64];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int e = 0; e < D / 64; ++e) acc[e] += v[i][e] * wc[i];
    }
    const int col0 = (hk * a.group + gq) * D;
#pragma unroll
    for (int e = 0; e < D / 64; ++e) {
        const float o = acc[e] / L;
        const u16 hi = f32_to_elem(o);
        const int col = col0 + lane + e * 64;
        a.out[operand_offset(m, col, a.out_tiles)] = hi;
        a.out[operand_offset(a.pair_rows + m, col, a.out_tiles)] = f32_to_elem(o - elem_to_f32(hi));
    }
}

template <int D, int MTW, int NWV>
__global__ __launch_bounds__(NWV * 64) void attn_partial_kernel(AttnArgs a) {
    constexpr int KS = D / 32;  // MFMA K steps of the QK^T product
    constexpr int DT = D / 16;  // 16-channel tiles of the PV product
    constexpr int NBUF = NWV / 2;
    __shared__ f32x4 lds_o[NBUF][MTW * DT * 64];
    __shared__ float lds_ml[NBUF][MTW][2][16];

    const int cb = blockIdx.x, hk = blockIdx.y, mg = blockIdx.z;
    // scalar wave index: MFMA ignores the EXEC mask, so all control flow around it must be wave-uniform
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;
    const int MQ = a.plan.M * a.group;

    // Visibility of draft slots, branch-free: with mk = key - P, row m sees mk < R (prefix and root)
    // and vis_lo <= mk <= vis_hi (its own sequence up to itself).
    elem8 qf[MTW][KS], ql[MTW][KS];
    int vis_lo[MTW], vis_hi[MTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        // query operand (B of S^T = K Q^T): column c of tile mt is pair r = (row m, head gq of the group)
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

    const u16* kbase = a.kc + (size_t)hk * a.max_seq * D + lane * 8;  // tiles are contiguous: lane l reads bytes 16*l ..
    const u16* vbase = a.vc + (size_t)hk * a.max_seq * D + lane * 8;
    const int b0 = (cb * NWV + wave) * a.blocks_per_wave;
    int nb = (a.Ktot + 31) / 32 - b0;  // this wave's blocks
    nb = nb < 0 ? 0 : (nb > a.blocks_per_wave ? a.blocks_per_wave : nb);

    // K and V^T tiles of one 32-key block, stored in MFMA operand layout.  S^T tile t, MFMA row 4g'+i' is
    // key kb + 8g' + 4t + i'; V^T operand dt is (channel dt*16 + c, keys kb + 8g .. +8).  Slots of the block at or
    // beyond Ktot may hold anything: their scores are replaced by -inf (a select), their values zeroed.
    elem8 kf[2][2][KS], vf[2][DT];  // double buffered: the next block is loaded while this one is used
    auto load_k = [&](int buf, int kb) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[buf][t][ks] = load_frag_stream(kbase + ((size_t)((kb >> 5) * 2 + t) * KS + ks) * 512);
    };
    auto load_v = [&](int buf, int kb) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) vf[buf][dt] = load_frag_stream(vbase + ((size_t)(kb >> 5) * DT + dt) * 512);
    };
    // scores of block kb (buffer buf), then request the next block's values (kb_next < 0: none), then
    // softmax and P V; the next block's keys were requested before the call
    auto use_block = [&](int buf, int kb, int kb_next) {
        const bool tail = kb + 32 > a.Ktot;      // slots at or beyond Ktot may hold anything: zero their V
        const bool masked = kb + 32 > a.plan.P;  // block touches draft slots or the end
        if (tail) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                Frag8 f;
                f.v = vf[buf][dt];
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (kb + g * 8 + j >= a.Ktot) f.h[j] = 0;
                vf[buf][dt] = f.v;
            }
        }
        float scs[MTW][8];
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16(kf[buf][t][ks], ql[mt][ks], acc);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16(kf[buf][t][ks], qf[mt][ks], acc);
#pragma unroll
                for (int i = 0; i < 4; ++i) scs[mt][t * 4 + i] = acc[i] * a.scale_log2;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (kb_next >= 0) load_v(buf ^ 1, kb_next);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
            float* sc = scs[mt];
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
            float pw[8], ps = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                pw[j] = exp2f(sc[j] - m_safe);
                ps += pw[j];
            }
            split_elem8(pw, pf.q, pl.q);
            l_run[mt] = l_run[mt] * alpha + ps;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                f32x4 acc = o[mt][dt] * alpha;
                acc = mfma16(vf[buf][dt], pl.v, acc);
                o[mt][dt] = mfma16(vf[buf][dt], pf.v, acc);
            }
        }
    };
    if (nb > 0) {
        load_k(0, b0 * 32);
        load_v(0, b0 * 32);
    }
    for (int ib = 0; ib < nb; ib += 2) {  // two blocks per trip so that the buffer index is static
        const int kb0 = (b0 + ib) * 32;
        const bool more1 = ib + 1 < nb, more2 = ib + 2 < nb;
        if (more1) load_k(1, kb0 + 32);
        __builtin_amdgcn_sched_barrier(0);
        use_block(0, kb0, more1 ? kb0 + 32 : -1);
        if (more1) {
            if (more2) load_k(0, kb0 + 64);
            __builtin_amdgcn_sched_barrier(0);
            use_block(1, kb0 + 32, more2 ? kb0 + 64 : -1);
        }
    }
    // lane-group partial sums -> row sums (max is already uniform across lane groups)
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        l_run[mt] += __shfl_xor(l_run[mt], 16, 64);
        l_run[mt] += __shfl_xor(l_run[mt], 32, 64);
    }

    // ---- merge the waves through LDS in a fixed binary tree: wave w + s -> wave w for s = NWV/2 .. 1
#pragma unroll
    for (int s = NWV / 2; s >= 1; s >>= 1) {
        if (wave >= s && wave < 2 * s) {
            const int buf = wave - s;
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) lds_o[buf][(mt * DT + dt) * 64 + lane] = o[mt][dt];
                if (g == 0) {
                    lds_ml[buf][mt][0][c] = m_run[mt];
                    lds_ml[buf][mt][1][c] = l_run[mt];
                }
            }
        }
        __syncthreads();
        if (wave < s) {
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) {
                const float mo = lds_ml[wave][mt][0][c], lo = lds_ml[wave][mt][1][c];
                const float mn = fmaxf(m_run[mt], mo);
                const float ms = mn == -INFINITY ? 0.f : mn;
                const float sa = exp2f(m_run[mt] - ms), sb = exp2f(mo - ms);
                m_run[mt] = mn;
                l_run[mt] = l_run[mt] * sa + lo * sb;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
                    o[mt][dt] = o[mt][dt] * sa + lds_o[wave][(mt * DT + dt) * 64 + lane] * sb;
            }
        }
        __syncthreads();
    }
    if (wave != 0) return;
    // wave 0 holds the chunk's result: lane (c, g) has O[r = c][dt*16 + 4g .. +4].  A head that is one
    // chunk is normalised and stored right away (bf16 pairs into the O projection's operand buffer);
    // otherwise the chunk partial goes to scratch for attn_combine_kernel.
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const int r = (mg * MTW + mt) * 16 + c;
        if (r >= MQ) continue;
        if (a.nchunks == 1) {
            const int m = r / a.group, col0 = (hk * a.group + r % a.group) * D;
            const float inv = 1.0f / l_run[mt];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float v = o[mt][dt][i] * inv;
                    const u16 hi = f32_to_elem(v);
                    const int col = col0 + dt * 16 + g * 4 + i;
                    a.out[operand_offset(m, col, a.out_tiles)] = hi;
                    a.out[operand_offset(a.pair_rows + m, col, a.out_tiles)] = f32_to_elem(v - elem_to_f32(hi));
                }
        } else {
            float* pp = a.part + (((size_t)hk * a.mq_pad + r) * a.nchunks + cb) * (D + 4);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4*>(pp + dt * 16 + g * 4) = o[mt][dt];
            if (g == 0) {
                pp[D] = m_run[mt];
                pp[D + 1] = l_run[mt];
            }
        }
    }
}

// Short contexts (at most 8 * BATCH blocks of 32 keys, up to 16 query rows per kv head): the whole head
// in one workgroup of eight waves, no loop.  A wave requests the keys of ALL its blocks and the values
// of the first one at once, forms every score, requests the remaining values into the registers the
// keys just left, does one plain softmax over its keys and the P V products; then the waves are merged
// through LDS in one step and every wave writes one 16-channel tile of the normalised output.  One memory latency for the keys and
// one for the values, instead of one per block.
template <int D, int BATCH>
__global__ __launch_bounds__(512) void attn_small_kernel(AttnArgs a) {
    constexpr int KS = D / 32, DT = D / 16, NWV = 8;
    __shared__ f32x4 lds_o[NWV][DT * 64];
    __shared__ float lds_ml[NWV][2][16];

    const int hk = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int c = lane & 15, g = lane >> 4;
    const int MQ = a.plan.M * a.group;

    const int r = c;  // column c of the one query tile is pair r = (row m, head gq of the group)
    const bool ok = r < MQ;
    const int m = ok ? r / a.group : 0, gq = ok ? r % a.group : 0;
    const int R = a.plan.R;
    const int vis_lo = !ok ? 0x7fffffff : (m < R ? 0 : R + ((m - R) / a.plan.k) * a.plan.k);
    const int vis_hi = ok ? m : -1;
    elem8 qf[KS], ql[KS];
    {
        const u16* qp = a.q + (size_t)m * a.ldq + (hk * a.group + gq) * D + g * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            Frag8 f;
            f.q = ok ? *reinterpret_cast<const u32x4*>(qp + ks * 32) : u32x4{0u, 0u, 0u, 0u};
            qf[ks] = f.v;
            f.q = ok ? *reinterpret_cast<const u32x4*>(qp + a.q_plane + ks * 32) : u32x4{0u, 0u, 0u, 0u};
            ql[ks] = f.v;
        }
    }
    const u16* kbase = a.kc + (size_t)hk * a.max_seq * D + lane * 8;
    const u16* vbase = a.vc + (size_t)hk * a.max_seq * D + lane * 8;
    const int NB = (a.Ktot + 31) / 32;
    // block b of this wave is global block wave + 8*b (round-robin keeps the waves within one block of each other)
    int nb = (NB - wave + NWV - 1) / NWV;
    nb = nb < 0 ? 0 : nb;

    elem8 kf[BATCH][2][KS], vf[BATCH][DT];
    auto load_v = [&](int b) {
        const int kb = (wave + NWV * b) * 32;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) vf[b][dt] = load_frag_stream(vbase + ((size_t)(kb >> 5) * DT + dt) * 512);
    };
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        if (b < nb) {
            const int blk = wave + NWV * b;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) kf[b][t][ks] = load_frag_stream(kbase + ((size_t)(blk * 2 + t) * KS + ks) * 512);
        }
    }
    if (nb > 0) load_v(0);
    __builtin_amdgcn_sched_barrier(0);

    float sc[BATCH][8];
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
#pragma unroll
        for (int j = 0; j < 8; ++j) sc[b][j] = -INFINITY;
        if (b < nb) {
            const int kb = (wave + NWV * b) * 32;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16(kf[b][t][ks], ql[ks], acc);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16(kf[b][t][ks], qf[ks], acc);
#pragma unroll
                for (int i = 0; i < 4; ++i) sc[b][t * 4 + i] = acc[i] * a.scale_log2;
            }
            if (kb + 32 > a.plan.P) {  // block touches draft slots or the end
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int mk = kb + g * 8 + j - a.plan.P;
                    const bool vis = (mk < R) | ((mk >= vis_lo) & (mk <= vis_hi));
                    sc[b][j] = vis ? sc[b][j] : -INFINITY;
                }
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int b = 1; b < BATCH; ++b)
        if (b < nb) load_v(b);
    __builtin_amdgcn_sched_barrier(0);

    // one softmax over all keys of this wave
    float mx = -INFINITY;
#pragma unroll
    for (int b = 0; b < BATCH; ++b)
#pragma unroll
        for (int j = 0; j < 8; ++j) mx = fmaxf(mx, sc[b][j]);
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_safe = mx == -INFINITY ? 0.f : mx;
    float m_run = mx, l_run = 0.f;
    f32x4 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int b = 0; b < BATCH; ++b) {
        if (b < nb) {
            const int kb = (wave + NWV * b) * 32;
            if (kb + 32 > a.Ktot) {  // slots at or beyond Ktot may hold anything: zero their V
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    Frag8 f;
                    f.v = vf[b][dt];
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (kb + g * 8 + j >= a.Ktot) f.h[j] = 0;
                    vf[b][dt] = f.v;
                }
            }
            Frag8 pf, pl;  // softmax weights as bf16 pairs (hi + lo)
            float pw[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                pw[j] = exp2f(sc[b][j] - m_safe);
                l_run += pw[j];
            }
            split_elem8(pw, pf.q, pl.q);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                o[dt] = mfma16(vf[b][dt], pl.v, o[dt]);
                o[dt] = mfma16(vf[b][dt], pf.v, o[dt]);
            }
        }
    }
    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);

    // Merge of the eight waves in one step: every wave leaves its unnormalised output, maximum and sum in LDS;
    // after one barrier wave w combines channel tile w of all eight (in wave order), normalises and stores it.
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) lds_o[wave][dt * 64 + lane] = o[dt];
    if (g == 0) {
        lds_ml[wave][0][c] = m_run;
        lds_ml[wave][1][c] = l_run;
    }
    __syncthreads();
    if (wave >= DT || !ok) return;
    float mall = lds_ml[0][0][c];
#pragma unroll
    for (int w = 1; w < NWV; ++w) mall = fmaxf(mall, lds_ml[w][0][c]);
    float L = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < NWV; ++w) {
        const float mw = lds_ml[w][0][c];
        const float sw = mw == -INFINITY ? 0.f : exp2f(mw - mall);
        L += lds_ml[w][1][c] * sw;
        acc += lds_o[w][wave * 64 + lane] * sw;
    }
    const int col0 = (hk * a.group + gq) * D;
    const float inv = 1.0f / L;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float v = acc[i] * inv;
        const u16 hi = f32_to_elem(v);
        const int col = col0 + wave * 16 + g * 4 + i;
        a.out[operand_offset(m, col, a.out_tiles)] = hi;
        a.out[operand_offset(a.pair_rows + m, col, a.out_tiles)] = f32_to_elem(v - elem_to_f32(hi));
    }
}

// Many query rows per kv head (more than two 16-row query tiles: many draft rows and/or a large GQA
// group).  The kernels above give every wave its own keys and ALL query tiles, which does not fit the
// registers beyond two tiles, so more tiles meant more workgroups re-reading the same keys.  Here it is
// the other way round: a workgroup takes one (kv head, key chunk); each 32-key block of K and V^T is put
// in LDS once, in MFMA operand layout (the same 1 KiB tiles the other kernels load straight into
// registers), and each of the NWV consumer waves owns MTW query tiles and runs over all blocks of the
// chunk, so nothing is merged between waves.  One extra wave does nothing but move the blocks: 16-byte
// global -> LDS loads (no registers, no LDS store instructions) into a ring of three buffers, two blocks
// ahead of the MFMAs; its barriers are bare s_barrier instructions behind a counted wait.  One barrier per
// block hands a filled buffer over and takes a drained one back.
//
// With few query tiles (KSPLIT > 1) the NWV consumer waves are KSPLIT teams of TW = NWV / KSPLIT waves and a ring stage
// holds KSPLIT blocks: team z takes block z of every stage for the workgroup's TW query tiles, so that every SIMD holds
// KSPLIT waves whose matrix, vector and LDS instructions overlap; the teams' softmax states are merged in team order
// through LDS at the end (the same rescaled sum the chunk merge uses).
// 2^x by the hardware instruction alone: results below the normal range come out as zero, which is all a softmax weight
// that small amounts to; 2^0 is exactly 1 and 2^-inf exactly 0.
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

template <int N>
__device__ __forceinline__ void wait_vector_loads_but() {  // vmcnt(N); expcnt and lgkmcnt fields at their maxima
    static_assert(N >= 0 && N <= 63, "the memory counter has six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

template <int D, int MTW, int NWV, int KSPLIT = 1>
__global__ __launch_bounds__((NWV + 1) * 64) void attn_shared_kernel(AttnArgs a) {
    constexpr int KS = D / 32, DT = D / 16;
    constexpr int KT = 2 * KS;      // K tiles per block (2 key halves x KS)
    constexpr int TILES = KT + DT;  // 1 KiB tiles per block
    constexpr int NBUF = 3;
    constexpr int TW = NWV / KSPLIT;  // query-tile waves per team
    constexpr int STL = KSPLIT * TILES;  // tiles per ring stage: one block for every team
    static_assert(STL <= 63, "a stage's loads fit the producer's memory counter");
    static_assert(NWV % KSPLIT == 0 && (KSPLIT == 1 || MTW == 1), "teams of equal size; one query tile per wave when the blocks are dealt to teams");
    __shared__ u32x4 lds_kv[NBUF][STL * 64];
    __shared__ f32x4 lds_team_o[KSPLIT > 1 ? (KSPLIT - 1) * TW * DT * 64 : 1];
    __shared__ float lds_team_ml[KSPLIT > 1 ? (KSPLIT - 1) * TW * 2 * 64 : 1];

    const int cb = blockIdx.x, hk = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;  // scalar: MFMA ignores EXEC
    const int c = lane & 15, g = lane >> 4;
    const int NB = (a.Ktot + 31) / 32;
    const int b0 = cb * a.blocks_per_wave;  // here: blocks per chunk
    int nb = NB - b0;
    nb = nb < 0 ? 0 : (nb > a.blocks_per_wave ? a.blocks_per_wave : nb);
    // Row groups in reverse launch order: workgroups start in index order, and the late rows of a prompt chunk see the
    // most keys, so the longest-running groups go first.
    const int zg = (int)(gridDim.z - 1 - blockIdx.z);
    {
        // No row sees a key behind its own slot: the blocks behind the slot of this workgroup's last query row
        // are masked for all of its rows and are left out (a prompt chunk's early rows skip the chunk's late keys).
        const int r_last = min(a.plan.M * a.group, (zg + 1) * TW * MTW * 16) - 1;
        const int nb_vis = (a.plan.P + r_last / a.group) / 32 + 1 - b0;
        nb = nb_vis < nb ? (nb_vis < 0 ? 0 : nb_vis) : nb;
    }

    const int nst = (nb + KSPLIT - 1) / KSPLIT;  // ring stages
    if (wave == NWV) {
        // ---- producer.  The cache stores the tiles as they are needed (see k_cache_offset / v_cache_offset):
        // tile j < KT of a block is K tile (t = j / KS, ks = j % KS), otherwise V^T tile dt = j - KT; each is 1 KiB,
        // lane l takes bytes 16*l ..
        const u16* kbase = a.kc + (size_t)hk * a.max_seq * D + lane * 8;
        const u16* vbase = a.vc + (size_t)hk * a.max_seq * D + lane * 8;
        auto issue = [&](int st) {  // stage st: blocks st * KSPLIT .. + KSPLIT of the chunk, as far as it has them
            u32x4* dst = lds_kv[st % NBUF];
#pragma unroll
            for (int z = 0; z < KSPLIT; ++z) {
                const int ib = st * KSPLIT + z;
                if (ib >= nb) break;  // wave-uniform
                const int blk = b0 + ib;
#pragma unroll
                for (int j = 0; j < TILES; ++j) {
                    const u16* src = j < KT ? kbase + ((size_t)blk * KT + j) * 512 : vbase + ((size_t)blk * DT + (j - KT)) * 512;
                    // cache policy 2: the non-temporal hint (every key and value byte is read once per pass)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                                     (__attribute__((address_space(3))) void*)(dst + (z * TILES + j) * 64), 16, 0, 2);
                }
            }
        };
        // Only blocks of the chunk are requested, so the wait before a hand-over counts the blocks of the one stage that
        // may still be in flight: vmcnt(blocks * TILES), everything older has landed (expcnt, lgkmcnt fields at their maxima).
        static_assert(KSPLIT <= 2, "the waits below know stages of one or two blocks");
        auto wait_all_but_stage = [&](int st) {
            const int blocks = st < nst ? min(KSPLIT, nb - st * KSPLIT) : 0;
            if (blocks == 0) wait_vector_loads_but<0>();
            else if (blocks == 1) wait_vector_loads_but<TILES>();
            else wait_vector_loads_but<2 * TILES>();
        };
        if constexpr (NWV == 4) {
            // Up to two query tiles per kv head: the first two stages are requested without a branch (blocks past the chunk
            // or the context repeat the last block of the context and are not used).  Behind a branch around global -> LDS
            // loads the compiler waits for everything in flight, so stage 1 is otherwise requested only after stage 0 has
            // landed.  Measured on whole steps: 3.538 -> 3.517 ms at two tiles (32 rows, 32 heads), but 4.600 -> 4.607 ms
            // at four tiles and 5.088 -> 5.096 ms at sixteen, where the kernel alone is faster too: those keep the branches.
            auto issue_unconditionally = [&](int st) {
                u32x4* dst = lds_kv[st % NBUF];
#pragma unroll
                for (int z = 0; z < KSPLIT; ++z) {
                    const int blk = min(b0 + st * KSPLIT + z, NB - 1);
#pragma unroll
                    for (int j = 0; j < TILES; ++j) {
                        const u16* src = j < KT ? kbase + ((size_t)blk * KT + j) * 512 : vbase + ((size_t)blk * DT + (j - KT)) * 512;
                        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                                         (__attribute__((address_space(3))) void*)(dst + (z * TILES + j) * 64), 16, 0, 2);
                    }
                }
            };
            issue_unconditionally(0);
            issue_unconditionally(1);
            wait_vector_loads_but<KSPLIT * TILES>();  // stage 0 has landed
        } else {
            if (nst > 0) issue(0);
            if (nst > 1) issue(1);
            wait_all_but_stage(1);  // stage 0 has landed
        }
        __builtin_amdgcn_s_barrier();
        for (int st = 0; st < nst; ++st) {
            if (st + 2 < nst) issue(st + 2);  // its buffer was drained in iteration st - 1
            wait_all_but_stage(st + 2);       // stage st + 1 has landed
            __builtin_amdgcn_s_barrier();
        }
        if (KSPLIT > 1) __builtin_amdgcn_s_barrier();  // the teams' hand-over
        return;
    }

    // ---- consumers
    const int MQ = a.plan.M * a.group;
    const int team = wave / TW, tw = wave - team * TW;
    const int tile0 = (zg * TW + tw) * MTW;  // first query tile of this wave
    elem8 qf[MTW][KS], ql[MTW][KS];
    int vis_lo[MTW], vis_hi[MTW];
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        const int r = (tile0 + mt) * 16 + c;
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
    auto use_block = [&](const u32x4* buf, int kb) {
        const bool masked = kb + 32 > a.plan.P;  // block touches draft slots or the end
        const bool tail = kb + 32 > a.Ktot;      // slots at or beyond Ktot may hold anything: zero their V
        auto frag = [&](int j) {
            Frag8 f;
            f.q = buf[j * 64 + lane];
            return f;
        };
        float scs[MTW][8];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            elem8 kf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[ks] = frag(t * KS + ks).v;
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) {  // lo and hi query parts into one accumulator; the scale comes with the exponent
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    acc = mfma16(kf[ks], ql[mt][ks], acc);
                    acc = mfma16(kf[ks], qf[mt][ks], acc);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) scs[mt][t * 4 + i] = acc[i];
            }
        }
        Frag8 pf[MTW], pl[MTW];
        float alpha[MTW];
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt) {
            float* sc = scs[mt];
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
            const float m_new = fmaxf(m_run[mt], bm * a.scale_log2);  // the running maximum is kept in scaled units
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            alpha[mt] = exp2_raw(m_run[mt] - m_safe);
            m_run[mt] = m_new;
            float pw[8], ps = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                pw[j] = exp2_raw(fmaf(sc[j], a.scale_log2, -m_safe));
                ps += pw[j];
            }
            split_elem8(pw, pf[mt].q, pl[mt].q);  // softmax weights as bf16 pairs (hi + lo)
            l_run[mt] = l_run[mt] * alpha[mt] + ps;
            // the running maximum rarely moves after the first blocks: rescale only when some row's did
            if (__ballot(alpha[mt] != 1.0f) != 0) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) o[mt][dt] = o[mt][dt] * alpha[mt];
            }
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            Frag8 vf = frag(KT + dt);
            if (tail) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (kb + g * 8 + e >= a.Ktot) vf.h[e] = 0;
            }
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) {
                f32x4 acc = mfma16(vf.v, pl[mt].v, o[mt][dt]);
                o[mt][dt] = mfma16(vf.v, pf[mt].v, acc);
            }
        }
    };

    // No row of this wave sees a key behind the slot of the wave's last query row: such blocks are masked for all of its
    // rows, so the wave leaves out their products and softmax (a prompt chunk's early rows against the chunk's late
    // keys: causal attention per query tile, not only per workgroup) and only keeps the ring's pace.
    const int r_wave_last = min(MQ, (tile0 + MTW) * 16) - 1;
    const int kb_last = r_wave_last >= 0 ? a.plan.P + r_wave_last / a.group : -1;  // key slot of that row
    __syncthreads();  // block 0 is in LDS
    for (int st = 0; st < nst; ++st) {
        const int ib = st * KSPLIT + team;  // this team's block of the stage
        const int kb = (b0 + ib) * 32;
        if (ib < nb && kb <= kb_last) use_block(lds_kv[st % NBUF] + team * TILES * 64, kb);  // wave-uniform
        __syncthreads();  // stage st + 1 is in LDS; stage st's buffer may be refilled
    }
    if constexpr (KSPLIT > 1) {
        // teams 1 .. KSPLIT-1 hand their states (running maximum, this lane's part of the sum, output) to team 0
        if (team > 0) {
            const int slot = (team - 1) * TW + tw;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) lds_team_o[(slot * DT + dt) * 64 + lane] = o[0][dt];
            lds_team_ml[(slot * 2 + 0) * 64 + lane] = m_run[0];
            lds_team_ml[(slot * 2 + 1) * 64 + lane] = l_run[0];
        }
        __syncthreads();
        if (team > 0) return;
#pragma unroll
        for (int z = 1; z < KSPLIT; ++z) {  // team order
            const int slot = (z - 1) * TW + tw;
            const float mz = lds_team_ml[(slot * 2 + 0) * 64 + lane], lz = lds_team_ml[(slot * 2 + 1) * 64 + lane];
            const float m_new = fmaxf(m_run[0], mz);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float s0 = exp2f(m_run[0] - m_safe), sz = exp2f(mz - m_safe);  // exp2(-inf) = 0: an empty state adds nothing
            m_run[0] = m_new;
            l_run[0] = l_run[0] * s0 + lz * sz;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[0][dt] = o[0][dt] * s0 + lds_team_o[(slot * DT + dt) * 64 + lane] * sz;
        }
    }

#pragma unroll
    for (int mt = 0; mt < MTW; ++mt) {
        l_run[mt] += __shfl_xor(l_run[mt], 16, 64);
        l_run[mt] += __shfl_xor(l_run[mt], 32, 64);
        const int r = (tile0 + mt) * 16 + c;
        if (r >= MQ) continue;
        if (a.nchunks == 1) {
            const int m = r / a.group, col0 = (hk * a.group + r % a.group) * D;
            const float inv = 1.0f / l_run[mt];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float v = o[mt][dt][i] * inv;
                    const u16 hi = f32_to_elem(v);
                    const int col = col0 + dt * 16 + g * 4 + i;
                    a.out[operand_offset(m, col, a.out_tiles)] = hi;
                    a.out[operand_offset(a.pair_rows + m, col, a.out_tiles)] = f32_to_elem(v - elem_to_f32(hi));
                }
        } else {
            float* pp = a.part + (((size_t)hk * a.mq_pad + r) * a.nchunks + cb) * (D + 4);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4*>(pp + dt * 16 + g * 4) = o[mt][dt];
            if (g == 0) {
                pp[D] = m_run[mt];
                pp[D + 1] = l_run[mt];
            }
        }
    }
}

// Merge of the chunk partials when a head was split over several workgroups: one wave per (row, head).
template <int D>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);  // four waves, four rows
    if (r < a.plan.M * a.group) attn_merge_row<D>(a, blockIdx.y, r, threadIdx.x & 63);
}

