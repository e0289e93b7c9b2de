// Skinny weight-streaming products y = x W^T for M <= 80 rows (the projections of the target
// pass, Alg. 1 right column).  The weights are read exactly once from HBM, straight into MFMA
// operand registers; the few activation rows are re-read from L2 by every workgroup.
//
// Streaming layout.  Both operands are stored in MFMA-tile order: a tile of 16 rows x 32 columns
// (one MFMA operand, 1 KiB) is contiguous, lane l's eight bf16 values at byte 16*l, i.e.
//     tile[(l % 16)][8 * (l / 16) + j]   at element   l * 8 + j        (l = 0..63, j = 0..7)
// and the K/32 tiles of a 16-row band follow each other.  A wave therefore reads its band of the
// weights as one linear stream, 1 KiB per load instruction, eight full cache lines at a time; with
// row-major weights the same load touches sixteen half lines and costs a third of the bandwidth.
// Weights are repacked once at load time (duo_pack.h); activations are written in this layout by
// the kernels that produce them ([k step][row tile][lane][8]).
//
// Work split: a workgroup owns NT bands of 16 weight rows and the whole K range; its NW waves
// take the K steps round-robin in groups of GRP, keep PF steps of loads in flight, and their partial
// sums are added in wave order through LDS (deterministic, no float atomics).  NW = 1 (one wave per
// workgroup, no partial sums) is used whenever the matrix has enough bands to fill the chip.  The
// epilogue functor decides what happens to the sums (plain store, residual add, SwiGLU, rotary
// embedding + KV-cache scatter).
//
// Activation precision: an activation a is carried as a bf16 pair (hi, lo) with hi = bf16(a),
// lo = bf16(a - hi), i.e. 16 mantissa bits.  The pair occupies two ROWS of the MFMA A operand:
// row m holds hi, row m + pair_rows holds lo, and the epilogue adds the two output rows.  For the
// common M <= 8 case both halves fit the one 16-row tile an MFMA needs anyway, so the extra
// precision costs nothing; a single bf16 per activation would leave rounding noise of ~0.1 in the
// logits of a 32-layer model.
#pragma once
#include "duo_common.h"

// element offset of (row r, column k) in an operand buffer of MT row tiles
__device__ __forceinline__ size_t operand_offset(int r, int k, int MT) {
    return ((size_t)((k >> 5) * MT + (r >> 4)) * 64 + ((k & 31) >> 3) * 16 + (r & 15)) * 8 + (k & 7);
}

// RMSNorm without a kernel of its own.  The producer of the residual stream (embedding gather or a
// residual projection) stores, next to x, the operand u = x * gain as bf16 pairs and, per row and per
// 16-column tile, the partial sum of x^2.  The consuming projection multiplies its output row m by
//     rs[m] = 1 / sqrt(sum of the partials / d + eps),
// which is the same product: (x * rs * gain) W^T = rs * ((x * gain) W^T).  The partials are added in
// a fixed order, identically in every workgroup.
struct RowScale {
    const float* part;  // [rows][n_part] partial sums of squares, nullptr: operand is not normalised
    int n_part;         // multiple of 4, at most 512
    float inv_d, eps;
    // [rows][FULL_PARTS] sums of squares over FULL_PARTS equal column ranges of the row (unused ranges hold zero) when
    // the producer was a few workgroups per row, else nullptr
    const float* full;
    static constexpr int FULL_PARTS = 8;
    __device__ __forceinline__ float full_row(int m) const {  // fixed order
        const f32x4 a = *reinterpret_cast<const f32x4*>(full + (size_t)m * FULL_PARTS);
        const f32x4 b = *reinterpret_cast<const f32x4*>(full + (size_t)m * FULL_PARTS + 4);
        return ((a.x + a.y) + (a.z + a.w)) + ((b.x + b.y) + (b.z + b.w));
    }
    static constexpr int MAXQ = 16;  // float4 loads per lane: 8 lanes x 16 x 4 = 512 partials per row
    // Eight rows at a time: lane = (row r0 + lane % 8, segment lane / 8); a lane adds its segment of the
    // row's partials in index order, the eight segments are then added by a fixed butterfly.  The loads
    // are issued together (load), the arithmetic comes later (reduce), so they overlap what lies between.
    __device__ __forceinline__ void load(f32x4 (&v)[MAXQ], int r0, int rows, int lane) const {
        const int m = r0 + (lane & 7), seg = lane >> 3;
        const int nq = n_part >> 2, len = (nq + 7) >> 3;
        const int b = seg * len, e = min(nq, b + len);
        const f32x4* row = reinterpret_cast<const f32x4*>(part + (size_t)(m < rows ? m : rows - 1) * n_part);
#pragma unroll
        for (int q = 0; q < MAXQ; ++q) {  // unconditional, index clamped into the row
            const int i = b + q;
            v[q] = row[i < e ? i : (e > 0 ? e - 1 : 0)];
        }
    }
    __device__ __forceinline__ void reduce(const f32x4 (&v)[MAXQ], float* out, int r0, int rows, int lane) const {
        const int seg = lane >> 3;
        const int nq = n_part >> 2, len = (nq + 7) >> 3;
        const int cnt = min(nq, seg * len + len) - seg * len;  // valid float4s of this lane's segment
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < MAXQ; ++q) {
            const float t = (v[q].x + v[q].y) + (v[q].z + v[q].w);
            s += q < cnt ? t : 0.f;
        }
        s += __shfl_xor(s, 8, 64);
        s += __shfl_xor(s, 16, 64);
        s += __shfl_xor(s, 32, 64);
        const int m = r0 + (lane & 7);
        if (seg == 0 && m < rows) out[m] = 1.0f / sqrtf(s * inv_d + eps);
    }
};

template <int MT, int NT, int NW, int PF, int GRP, class Epi, bool STREAM = true>
__global__ __launch_bounds__(NW * 64) void gemm_skinny_kernel(const u16* __restrict__ X, const u16* __restrict__ W, int K,
                                                               int quads, int pair_quads, RowScale rsc, Epi epi) {
    __shared__ f32x4 red[NW * MT * NT * 64];
    __shared__ float row_scale[MT * 16];
    const int tile = blockIdx.x;
    // the wave index must live in a scalar register: MFMA ignores the EXEC mask, so every branch
    // around an MFMA has to be a scalar (wave-uniform) branch, never lane predication
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int steps = K >> 5;

    const u16* wp[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) wp[t] = W + ((size_t)(tile * NT + t) * steps) * 512 + lane * 8;
    const u16* xp = X + lane * 8;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // K steps are dealt to the waves in groups of GRP consecutive steps
    const int groups = (steps + GRP - 1) / GRP;
    const int my_groups = (groups - wave + NW - 1) / NW;
    int ni = my_groups * GRP;  // this wave's steps (the last group of the matrix may be short)
    auto step_of = [&](int i) { return ((i / GRP) * NW + wave) * GRP + (i % GRP); };
    if (ni > 0 && step_of(ni - 1) >= steps) ni -= step_of(ni - 1) - steps + 1;

    // Software pipeline with PF register slots per operand.  Slot p always holds step i0 + p; a slot is
    // refilled right after the MFMAs that consumed it, so every slot keeps its registers for the whole
    // loop and the number of loads in flight behind any MFMA is the same in every iteration.  All loads
    // are unconditional (indices clamped to the wave's last step) and scheduling barriers keep the
    // compiler from regrouping them, so the wait before each MFMA group is for exactly one slot.
    elem8 bb[PF][NT], aa[PF][MT];
    auto load_slot = [&](int p, int i) {
        const int st = step_of(i);
#pragma unroll
        for (int t = 0; t < NT; ++t) bb[p][t] = STREAM ? load_frag_stream(wp[t] + (size_t)st * 512) : load_frag(wp[t] + (size_t)st * 512);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) aa[p][mt] = load_frag(xp + ((size_t)st * MT + mt) * 512);
    };
    auto mfma_slot = [&](int p) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[mt][t] = mfma16(aa[p][mt], bb[p][t], acc[mt][t]);
    };
    // What the epilogue will read from memory (residual values, gains, rotary factors) is requested now,
    // for the first output quad of each thread, so that its latency hides behind the weight stream.
    typename Epi::Pre pre;
    epi.arm();
    epi.prefetch(tile, min((int)threadIdx.x >> 4, quads - 1), threadIdx.x & 15, pre);  // every thread: no branch around loads
    // Per-row RMSNorm factors of the operand (see RowScale): the partial sums of the wave's first eight
    // rows are requested before the first weights and added up while those are in flight.
    // (compile-time for epilogues whose input takes no factors: every branch between the prefetch and the main loop is a
    // join at which the compiler waits for most of the prefetch)
    constexpr bool NORM = Epi::NORMALISED_INPUT;
    const int nrows = quads * 4;
    f32x4 rsv[RowScale::MAXQ];
    const bool rs_first = NORM && rsc.part && wave * 8 < nrows;
    if (rs_first) rsc.load(rsv, wave * 8, nrows, lane);
    __builtin_amdgcn_sched_barrier(0);
    if (ni > 0) {
#pragma unroll
        for (int p = 0; p < PF; ++p) load_slot(p, p < ni ? p : ni - 1);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (rs_first) rsc.reduce(rsv, row_scale, wave * 8, nrows, lane);
    if (NORM && rsc.part)
        for (int r0 = (wave + NW) * 8; r0 < nrows; r0 += NW * 8) {  // more than 8 * NW rows
            rsc.load(rsv, r0, nrows, lane);
            rsc.reduce(rsv, row_scale, r0, nrows, lane);
        }
    __builtin_amdgcn_sched_barrier(0);
    if (ni > 0) {
        int i0 = 0;
        for (; i0 + PF < ni; i0 += PF) {
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                mfma_slot(p);
                const int in = i0 + p + PF;
                load_slot(p, in < ni ? in : ni - 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int p = 0; p < PF; ++p) {  // drain: the last (up to PF) steps are already in the slots
            if (i0 + p < ni) mfma_slot(p);
            __builtin_amdgcn_sched_barrier(0);
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
            if (NORM && rsc.part) {
#pragma unroll
                for (int i = 0; i < 4; ++i) s[i] *= row_scale[qi * 4 + i];
            }
            v[t] = s;
        }
        epi.store(tile, qi, c, v, pre, idx == (int)threadIdx.x);
    }
}

// Variant for more than eight rows (M = 9..80, i.e. MH = 1..5 tiles of hi rows plus as many of lo rows).
// With that many rows the activation operand is no longer negligible next to the weights: every wave of the
// kernel above re-reads all 2*MH tiles of it per K step.  Here the NG consumer waves of a workgroup share it
// through LDS, each taking its own group of NT weight bands (every weight byte still goes from HBM straight
// into one wave's registers, PF steps ahead); hi and lo products accumulate into the same registers (for few
// tiles into separate ones, so that dependent MFMAs on one accumulator have others in between), and the
// epilogue runs straight from the accumulators.  The weights are the FIRST MFMA operand here, so a lane's quad is
// four consecutive columns of one output row and the epilogue stores vectors (store4).  The grid's y dimension
// splits K across workgroups for matrices with few bands (partial results, see EpiStoreF32).  All loads of
// the main loop are unconditional with clamped indices and invalid steps multiply by zero: no branches, so
// the counted waits stay exact.
//
// With HALF the operand is the single tile of up to eight rows (hi rows 0..7, lo rows 8..15 of the same tile),
// as the kernel above uses it, activations first (a lane's quad is four rows of one column); the two halves of the
// sums are then 32 lanes apart.
//
// One extra wave per workgroup does nothing but move the activation operand:
// wave NG copies the operand tiles of round r + 2 from global memory straight into a three-deep ring of
// LDS buffers (16-byte global -> LDS loads, no registers, no LDS store instructions) while the NG consumer
// waves stream their weight bands and compute on round r.  The consumers' memory counter then tracks the
// weight stream alone, PF steps ahead, and their registers hold weights and accumulators only.
// One barrier per round hands a filled buffer over and takes a drained one back.  Matrices with few bands
// put NK waves on each band group: they split the K steps of every round (NK * AG steps) between them and
// add their partial sums through LDS in wave order at the end.
template <int MH, int NT, int NG, int NK, int PF, int AG, class Epi, bool HALF = false, bool STREAM = true>
__global__ __launch_bounds__((NG * NK + 1) * 64) void gemm_wide_kernel(const u16* __restrict__ X, const u16* __restrict__ W,
                                                                      int K, int split_steps, int ntiles, int quads,
                                                                      RowScale rsc, Epi epi) {
    static_assert(!HALF || MH == 1, "the shared-tile layout holds at most eight rows");
    constexpr int MT = HALF ? 1 : 2 * MH, NC = NG * NK, NTH = (NC + 1) * 64;
    constexpr int RS = NK * AG;        // K steps per round
    constexpr int BUF = RS * MT * 64;  // 16-byte chunks per ring buffer (one round)
    constexpr int NBUF = 3;
    constexpr int L = RS * MT;  // global -> LDS loads per round
    constexpr int U = PF / AG;  // rounds per turn of the weight slots
    static_assert(PF % AG == 0 && AG % 2 == 0 && L <= 63, "slots cover whole rounds; a round's loads fit the memory counter");
    constexpr bool SEP = !HALF && MH * NT < 4;  // few tiles: separate lo accumulators
    constexpr int MA = SEP ? MT : MH;
    constexpr int RED = NK > 1 ? NC * MH * NT * 64 : 0;  // partial sums of the K-splitting waves (reuses the ring)
    static_assert(RED <= NBUF * BUF, "the partial sums fit the ring buffers");
    __shared__ u32x4 lds[NBUF * BUF];
    __shared__ float row_scale[MH * 16];
    // HALF, factors from partial sums (the producer of the rows was a one-kernel residual projection): the eight rows'
    // partial sums come in with the producer wave's first global -> LDS loads and every consumer wave adds them up for
    // itself once round 0 has landed, in the order RowScale::reduce uses.  Fetching them into registers at the top of the
    // kernel holds up the wave that does it, and with it the first hand-over, by a memory round trip (1.1 us of the Q/K/V
    // projection's 18.9 us at eight rows).
    constexpr int RAW16 = HALF ? 8 * 512 / 4 : 1;  // 16-byte pieces: eight rows of at most 512 partial sums
    __shared__ u32x4 part_raw[RAW16];
    __shared__ float row_scale_w[HALF ? NG * NK * 8 : 1];
    const bool raw_part = HALF && rsc.part && !rsc.full;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;  // scalar: MFMA ignores EXEC
    const int steps = K >> 5;
    const int k0 = blockIdx.y * split_steps;
    const int ns = min(steps - k0, split_steps);  // K steps of this split (the host makes it positive)
    const int rounds = (ns + RS - 1) / RS;
    const int rounds_run = (rounds + U - 1) / U * U;  // what the consumers' unrolled loop executes
    const u32x4* xg = reinterpret_cast<const u32x4*>(X) + (size_t)k0 * MT * 64 + lane;

    if (rsc.full) {
        for (int m = threadIdx.x; m < quads * 4; m += NTH) row_scale[m] = 1.0f / sqrtf(rsc.full_row(m) * rsc.inv_d + rsc.eps);
    } else if (rsc.part && !raw_part) {
        const int nrows = quads * 4;
        f32x4 rsv[RowScale::MAXQ];
        for (int r0 = wave * 8; r0 < nrows; r0 += (NC + 1) * 8) {
            rsc.load(rsv, r0, nrows, lane);
            rsc.reduce(rsv, row_scale, r0, nrows, lane);
        }
    }

    if (wave == NC) {
        // ---- producer: round r goes to ring buffer r % 3; steps past the end re-read the last step
        auto issue = [&](int r) {
            const int b = r % NBUF;
#pragma unroll
            for (int i = 0; i < L; ++i) {
                int st = r * RS + i / MT;
                st = st < ns ? st : ns - 1;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xg + ((size_t)st * MT + i % MT) * 64),
                                                 (__attribute__((address_space(3))) void*)(lds + b * BUF + i * 64), 16, 0, 0);
            }
        };
        // The barriers of this wave are bare s_barrier instructions behind a counted wait: a fence here would
        // wait for ALL outstanding loads, including the round just requested.  vmcnt(L) = everything but the
        // youngest round has landed in LDS (expcnt and lgkmcnt fields left at their maxima).
        constexpr int WAIT_ALL_BUT_ONE_ROUND = (L & 15) | ((L >> 4) << 14) | (7 << 4) | (15 << 8);
        if constexpr (HALF) {
            // older than every round: the first counted wait below covers them.  No branch around them (a join here makes
            // the compiler wait for everything in flight): without partial sums to fetch, the pieces re-read the operand.
            const int n16 = raw_part ? 2 * rsc.n_part : 64;  // eight rows x n_part floats
            const u32x4* src = raw_part ? reinterpret_cast<const u32x4*>(rsc.part) : reinterpret_cast<const u32x4*>(X);
#pragma unroll
            for (int c = 0; c < RAW16 / 64; ++c) {  // pieces past the end repeat the last one
                const int i = min(c * 64 + lane, n16 - 1);
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + i),
                                                 (__attribute__((address_space(3))) void*)(part_raw + c * 64), 16, 0, 0);
            }
        }
        issue(0);
        issue(1);
        __builtin_amdgcn_s_waitcnt(WAIT_ALL_BUT_ONE_ROUND & ~(15 << 8));  // and lgkmcnt(0): this wave's row scales are written
        __builtin_amdgcn_s_barrier();
        for (int r = 0; r < rounds_run; ++r) {
            issue(r + 2);  // its buffer was drained in round r - 1
            __builtin_amdgcn_s_waitcnt(WAIT_ALL_BUT_ONE_ROUND);  // round r + 1 has landed
            __builtin_amdgcn_s_barrier();
        }
        if (NK > 1) {  // the consumers reuse the ring for their partial sums: nothing may land in it any more
            __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));  // vmcnt(0)
            __builtin_amdgcn_s_barrier();                      // ring is quiet
            __builtin_amdgcn_s_barrier();                      // partial sums are written
        }
        return;
    }

    // ---- consumers: wave (ng, nk) takes band group ng and, of every round, the K steps nk * AG .. + AG
    const int ng = wave % NG, nk = wave / NG;
    const int tile_raw = blockIdx.x * NG + ng;
    const bool live = tile_raw < ntiles;
    const int tile = live ? tile_raw : ntiles - 1;
    const u16* wp[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) wp[t] = W + ((size_t)(tile * NT + t) * steps + k0) * 512 + lane * 8;
    f32x4 acc[MA][NT];
#pragma unroll
    for (int m = 0; m < MA; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    elem8 bb[PF][NT];
    elem8 af[2][MT];
    auto w_load = [&](int p, int i) {  // i-th step of this wave: round i / AG, position nk * AG + i % AG in it; clamped
        int ls = (i / AG) * RS + nk * AG + (i % AG);
        ls = ls < ns ? ls : ns - 1;
#pragma unroll
        for (int t = 0; t < NT; ++t) bb[p][t] = STREAM ? load_frag_stream(wp[t] + (size_t)ls * 512) : load_frag(wp[t] + (size_t)ls * 512);
    };
    auto a_frags = [&](int slot, int r, int w) {  // this wave's step w of round r
        const u32x4* ab = lds + (r % NBUF) * BUF + (nk * AG + w) * MT * 64 + lane;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            Frag8 f;
            f.q = ab[mt * 64];
            af[slot][mt] = f.v;
        }
    };
    typename Epi::Pre pre;
    epi.arm();
    const int first_mh = NK > 1 ? nk : 0;  // the first row tile this wave finishes
    if constexpr (HALF) epi.prefetch(tile, min(first_mh * 4 + (lane >> 4), quads - 1), lane & 15, pre);  // store4 takes none; every lane: no branch around loads
#pragma unroll
    for (int p = 0; p < PF; ++p) w_load(p, p);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();  // round 0 is in LDS, the row scales are written
    a_frags(0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    const float* rsp = row_scale;
    if constexpr (HALF) {
        if (raw_part) {  // LDS reads only: the weight stream's memory counter is not involved
            const int m = lane & 7, seg = lane >> 3;
            const int nq = rsc.n_part >> 2, len = (nq + 7) >> 3;
            const int b = seg * len, e = min(nq, b + len);
            const f32x4* row = reinterpret_cast<const f32x4*>(part_raw) + m * nq;
            f32x4 rsv[RowScale::MAXQ];
#pragma unroll
            for (int q = 0; q < RowScale::MAXQ; ++q) {
                const int i = b + q;
                rsv[q] = row[i < e ? i : (e > 0 ? e - 1 : 0)];
            }
            rsc.reduce(rsv, row_scale_w + wave * 8, 0, 8, lane);
            rsp = row_scale_w + wave * 8;
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    const elem8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int r0 = 0; r0 < rounds; r0 += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int r = r0 + u;  // may run past the last round: those steps multiply by zero
#pragma unroll
            for (int w = 0; w < AG; ++w) {
                const int p = u * AG + w;
                if (w + 1 < AG) a_frags((p + 1) & 1, r, w + 1);
                const bool valid = r * RS + nk * AG + w < ns;
                elem8 b[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) b[t] = valid ? bb[p][t] : zero;
                if constexpr (HALF) {  // activations first: a lane's quad is four rows of one column
#pragma unroll
                    for (int t = 0; t < NT; ++t) acc[0][t] = mfma16(af[p & 1][0], b[t], acc[0][t]);
                } else {  // weights first: a lane's quad is four consecutive columns of one row (vector stores)
#pragma unroll
                    for (int mh = 0; mh < MH; ++mh)
#pragma unroll
                        for (int t = 0; t < NT; ++t) acc[mh][t] = mfma16(b[t], af[p & 1][mh], acc[mh][t]);
#pragma unroll
                    for (int mh = 0; mh < MH; ++mh)
#pragma unroll
                        for (int t = 0; t < NT; ++t)
                            acc[SEP ? MH + mh : mh][t] = mfma16(b[t], af[p & 1][MH + mh], acc[SEP ? MH + mh : mh][t]);
                }
                w_load(p, (r + U) * AG + w);
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();  // round r + 1 is in LDS; round r's buffer may be refilled
            a_frags(0, r + 1, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // HALF: a lane's accumulator quad is rows 4*(lane/16) .. +3, column lane%16 of its tile (one output quad of the
    // epilogue's store).  Otherwise it is row 16*mh + lane%16 and columns 4*(lane/16) .. +3 (store4).
    auto finish = [&](int mh, f32x4 (&v)[NT], bool use_pre) {
        if constexpr (HALF) {  // rows 0..7 hold the hi sums, rows 8..15 (32 lanes further on) the lo sums; all lanes take part
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) v[t][i] += __shfl_xor(v[t][i], 32, 64);
            const int qi = mh * 4 + (lane >> 4);
            if (qi < quads) {
                if (rsc.part) {
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[t][i] *= rsp[qi * 4 + i];
                }
                epi.store(tile, qi, lane & 15, v, pre, use_pre);
            }
        } else {
            const int m = mh * 16 + (lane & 15);
            if (m < quads * 4) {
                if (rsc.part) {
                    const float rs = row_scale[m];
#pragma unroll
                    for (int t = 0; t < NT; ++t) v[t] = v[t] * rs;
                }
                epi.store4(tile, m, 4 * (lane >> 4), v);
            }
        }
    };
    if (NK == 1) {
        if (live) {  // wave-uniform
#pragma unroll
            for (int mh = 0; mh < MH; ++mh) {
                f32x4 v[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) v[t] = SEP ? acc[mh][t] + acc[MA - MH + mh][t] : acc[mh][t];
                finish(mh, v, mh == 0);
            }
        }
    } else {
        f32x4* red = reinterpret_cast<f32x4*>(lds);
        __syncthreads();  // the producer has seen its last load land: the ring is quiet
#pragma unroll
        for (int mh = 0; mh < MH; ++mh)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                red[((wave * MH + mh) * NT + t) * 64 + lane] = SEP ? acc[mh][t] + acc[MA - MH + mh][t] : acc[mh][t];
        __syncthreads();
        if (live) {
            for (int mh = nk; mh < MH; mh += NK) {  // K parts added in wave order
                f32x4 v[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    f32x4 sum = red[((ng * MH + mh) * NT + t) * 64 + lane];
#pragma unroll
                    for (int kk = 1; kk < NK; ++kk) sum += red[(((kk * NG + ng) * MH + mh) * NT + t) * 64 + lane];
                    v[t] = sum;
                }
                finish(mh, v, mh == nk);
            }
        }
    }
}

// ---- epilogues -------------------------------------------------------------------------------
// store(tile, qi, c, v): v[t][i] is the sum for row m = 4*qi + i, column c of tile slot t.
// store4(tile, m, c4, v): v[t][i] is the sum for row m, column c4 + i of tile slot t (c4 = 0, 4, 8, 12): what a
// lane holds when the weights are the first MFMA operand.  Four consecutive columns are 16 bytes of an fp32
// row and 8 bytes (half a 16-byte chunk) of a bf16 operand buffer, so the stores are vectors.
// arm(): called once by every consumer wave before the weight stream starts; an epilogue that depends on device
// state reads it here, so that its latency hides behind the stream.

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// four floats -> hi = bf16(x) and lo = bf16(x - hi), four bf16 values (8 bytes) each
__device__ __forceinline__ void split_elem4(const f32x4& x, u32x2& hi, u32x2& lo) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const uint32_t h = pack_elem2(x[2 * j], x[2 * j + 1]);
        hi[j] = h;
        lo[j] = pack_elem2(x[2 * j] - elem2_lo_f32(h), x[2 * j + 1] - elem2_hi_f32(h));
    }
}
__device__ __forceinline__ u32x2 pack_elem4(const f32x4& x) {
    return u32x2{pack_elem2(x[0], x[1]), pack_elem2(x[2], x[3])};
}

struct EpiStoreF32 {  // y[m][n] = sum ; band t of a workgroup covers rows (tile*NT + t)*16 .. +16 of W
    static constexpr const char* NAME = "EpiStoreF32";
    static constexpr bool NORMALISED_INPUT = true;
    int N, M, NT;
    float* Y;
    int ldy;
    size_t split_stride;  // elements between the outputs of two K splits (grid y); 0 when K is not split
    struct Pre {};
    __device__ __forceinline__ void arm() {}
    __device__ __forceinline__ void prefetch(int, int, int, Pre&) const {}
    template <int NTT>
    __device__ __forceinline__ void store(int tile, int qi, int c, const f32x4 (&v)[NTT], const Pre&, bool) const {
        float* y = Y + blockIdx.y * split_stride;
#pragma unroll
        for (int t = 0; t < NTT; ++t) {
            const int n = (tile * NT + t) * 16 + c;
            if (n >= N) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = qi * 4 + i;
                if (m < M) y[(size_t)m * ldy + n] = v[t][i];
            }
        }
    }
    template <int NTT>
    __device__ __forceinline__ void store4(int tile, int m, int c4, const f32x4 (&v)[NTT]) const {
        if (m >= M) return;
        float* y = Y + blockIdx.y * split_stride + (size_t)m * ldy;
#pragma unroll
        for (int t = 0; t < NTT; ++t) {
            const int n = (tile * NT + t) * 16 + c4;
            if (n + 3 < N && (ldy & 3) == 0) {
                *reinterpret_cast<f32x4*>(y + n) = v[t];
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (n + i < N) y[n + i] = v[t][i];
            }
        }
    }
};

// LM head of the verify step (Alg. 2 works on p = softmax(logits / T)): stores the fp32 logits like EpiStoreF32 and,
// from the same registers, the softmax statistics of every row over this tile's 16 * NT columns, in double: the max
// of z = logit / T and sum exp(z - max), or at T == 0 (the greedy limit) the largest logit and the lowest id that
// attains it.  parts [M][nparts][2], part index = tile; the sampling kernels merge a row's parts in index order.
struct EpiLogitsStats {
    static constexpr const char* NAME = "EpiLogitsStats";
    static constexpr bool NORMALISED_INPUT = true;
    int N, M, NT;
    float* Y;
    int ldy;
    double* parts;
    int nparts;
    double T;
    struct Pre {};
    __device__ __forceinline__ void arm() {}
    __device__ __forceinline__ void prefetch(int, int, int, Pre&) const {}
    // one row's statistics from this lane's `cnt` values z (ids id[]), combined over the lanes `masks` apart
    template <int CNT, int NMASK>
    __device__ __forceinline__ void row_stats(const float (&x)[CNT], const int (&id)[CNT], const int (&masks)[NMASK], bool writer,
                                              double* out) const {
        double mx = -INFINITY;
        if (T == 0.0) {
#pragma unroll
            for (int e = 0; e < CNT; ++e)
                if (id[e] < N) mx = fmax(mx, (double)x[e]);
#pragma unroll
            for (int q = 0; q < NMASK; ++q) mx = fmax(mx, __shfl_xor(mx, masks[q], 64));
            double first = 4.0e9;
#pragma unroll
            for (int e = 0; e < CNT; ++e)
                if (id[e] < N && (double)x[e] == mx) first = fmin(first, (double)id[e]);
#pragma unroll
            for (int q = 0; q < NMASK; ++q) first = fmin(first, __shfl_xor(first, masks[q], 64));
            if (writer) {
                out[0] = mx;
                out[1] = first;
            }
            return;
        }
        double z[CNT];
#pragma unroll
        for (int e = 0; e < CNT; ++e) {
            z[e] = (double)x[e] / T;
            if (id[e] < N) mx = fmax(mx, z[e]);
        }
#pragma unroll
        for (int q = 0; q < NMASK; ++q) mx = fmax(mx, __shfl_xor(mx, masks[q], 64));
        double sum = 0.0;
#pragma unroll
        for (int e = 0; e < CNT; ++e)
            if (id[e] < N) sum += exp(z[e] - mx);
#pragma unroll
        for (int q = 0; q < NMASK; ++q) sum += __shfl_xor(sum, masks[q], 64);
        if (writer) {
            out[0] = mx;
            out[1] = sum;
        }
    }
    // rows 4*qi .. +3, column c of each band: the tile's 16 columns sit in 16 consecutive lanes (all of them call this)
    template <int NTT>
    __device__ __forceinline__ void store(int tile, int qi, int c, const f32x4 (&v)[NTT], const Pre&, bool) const {
        const int masks[4] = {8, 4, 2, 1};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = qi * 4 + i;
            float x[NTT];
            int id[NTT];
#pragma unroll
            for (int t = 0; t < NTT; ++t) {
                x[t] = v[t][i];
                id[t] = (tile * NT + t) * 16 + c;
                if (m < M && id[t] < N) Y[(size_t)m * ldy + id[t]] = x[t];
            }
            row_stats<NTT, 4>(x, id, masks, c == 0 && m < M, parts + ((size_t)(m < M ? m : 0) * nparts + tile) * 2);
        }
    }
    // row m, columns c4 .. c4+3 of each band: the tile's columns sit in the four lanes 16 apart that share the row
    template <int NTT>
    __device__ __forceinline__ void store4(int tile, int m, int c4, const f32x4 (&v)[NTT]) const {
        if (m >= M) return;  // the four lanes of a row leave together
        float* y = Y + (size_t)m * ldy;
        float x[NTT * 4];
        int id[NTT * 4];
#pragma unroll
        for (int t = 0; t < NTT; ++t) {
            const int n = (tile * NT + t) * 16 + c4;
            if (n + 3 < N && (ldy & 3) == 0) {
                *reinterpret_cast<f32x4*>(y + n) = v[t];
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (n + i < N) y[n + i] = v[t][i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[t * 4 + i] = v[t][i];
                id[t * 4 + i] = n + i;
            }
        }
        const int masks[2] = {16, 32};
        row_stats<NTT * 4, 2>(x, id, masks, c4 == 0, parts + ((size_t)m * nparts + tile) * 2);
    }
};

// x[m][n] += sum (fp32 residual stream, each element owned by one workgroup).  The same thread then
// prepares the next RMSNorm (see RowScale): u = x * gain as a bf16 pair into the next projection's
// operand buffer, and the tile's partial sum of x^2 per row.  One band per workgroup (NT = 1).
struct EpiResidual {
    static constexpr const char* NAME = "EpiResidual";
    static constexpr bool NORMALISED_INPUT = false;  // its input is never an RMSNorm operand (attention output, SwiGLU output): the kernels compile the factors out
    int N, M;
    float* X;
    int ldx;
    const u16* gain;  // gain of the norm that follows
    u16* h;           // operand buffer of the next projection
    int pair_rows, h_tiles;
    float* ssq_part;  // [M][N/16]
    struct Pre {
        float x[4], g;
    };
    __device__ __forceinline__ void arm() {}
    __device__ __forceinline__ void prefetch(int tile, int qi, int c, Pre& p) const {
        // no branch around a load: behind a join the compiler waits for every load in flight, and the weight stream
        // would start a memory round trip late (rows past M re-read row M - 1 and are not used)
        const int n = tile * 16 + c;
        p.g = elem_to_f32(gain[n]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = qi * 4 + i;
            p.x[i] = X[(size_t)(m < M ? m : M - 1) * ldx + n];
        }
    }
    __device__ __forceinline__ void store(int tile, int qi, int c, const f32x4 (&v)[1], const Pre& p, bool use_pre) const {
        const int n = tile * 16 + c;
        const float gn = use_pre ? p.g : elem_to_f32(gain[n]);
        float sq[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = qi * 4 + i;
            sq[i] = 0.f;
            if (m < M) {
                const float xn = (use_pre ? p.x[i] : X[(size_t)m * ldx + n]) + v[0][i];
                X[(size_t)m * ldx + n] = xn;
                sq[i] = xn * xn;
                const float u = xn * gn;
                const u16 hi = f32_to_elem(u);
                h[operand_offset(m, n, h_tiles)] = hi;
                h[operand_offset(pair_rows + m, n, h_tiles)] = f32_to_elem(u - elem_to_f32(hi));
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // sum over the 16 columns of the tile (16 consecutive lanes)
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) sq[i] += __shfl_xor(sq[i], o, 64);
            const int m = qi * 4 + i;
            if (c == 0 && m < M) ssq_part[(size_t)m * (N >> 4) + tile] = sq[i];
        }
    }
    // All 64 lanes call this together; the lanes c4 = 0, 4, 8, 12 of one row are 16 lanes apart.
    __device__ __forceinline__ void store4(int tile, int m, int c4, const f32x4 (&v)[1]) const {
        const int n = tile * 16 + c4;
        float sq = 0.f;
        if (m < M) {
            float* xp = X + (size_t)m * ldx + n;
            const f32x4 xn = *reinterpret_cast<const f32x4*>(xp) + v[0];
            *reinterpret_cast<f32x4*>(xp) = xn;
            sq = (xn[0] * xn[0] + xn[1] * xn[1]) + (xn[2] * xn[2] + xn[3] * xn[3]);
            const u32x2 gb = *reinterpret_cast<const u32x2*>(gain + n);
            const f32x4 u = {xn[0] * elem2_lo_f32(gb[0]), xn[1] * elem2_hi_f32(gb[0]), xn[2] * elem2_lo_f32(gb[1]),
                             xn[3] * elem2_hi_f32(gb[1])};
            u32x2 hi, lo;
            split_elem4(u, hi, lo);
            *reinterpret_cast<u32x2*>(h + operand_offset(m, n, h_tiles)) = hi;
            *reinterpret_cast<u32x2*>(h + operand_offset(pair_rows + m, n, h_tiles)) = lo;
        }
        sq += __shfl_xor(sq, 16, 64);  // the tile's sixteen columns: four lanes, 16 apart
        sq += __shfl_xor(sq, 32, 64);
        if (c4 == 0 && m < M) ssq_part[(size_t)m * (N >> 4) + tile] = sq;
    }
};

// band 0 = gate rows tile*16.., band 1 = up rows tile*16..; act[m][n] = silu(gate) * up, written as a
// bf16 pair straight into the down projection's operand buffer (row m hi, row pair_rows + m lo)
struct EpiSwiGLU {
    static constexpr const char* NAME = "EpiSwiGLU";
    static constexpr bool NORMALISED_INPUT = true;
    int F, M;
    u16* act;
    int act_tiles, pair_rows;
    struct Pre {};
    __device__ __forceinline__ void arm() {}
    __device__ __forceinline__ void prefetch(int, int, int, Pre&) const {}
    __device__ __forceinline__ void store(int tile, int qi, int c, const f32x4 (&v)[2], const Pre&, bool) const {
        const int n = tile * 16 + c;
        if (n >= F) return;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = qi * 4 + i;
            if (m < M) {
                const float gate = v[0][i], up = v[1][i];
                const float a = gate / (1.f + expf(-gate)) * up;
                const u16 hi = f32_to_elem(a);
                act[operand_offset(m, n, act_tiles)] = hi;
                act[operand_offset(pair_rows + m, n, act_tiles)] = f32_to_elem(a - elem_to_f32(hi));
            }
        }
    }
    __device__ __forceinline__ void store4(int tile, int m, int c4, const f32x4 (&v)[2]) const {
        const int n = tile * 16 + c4;
        if (n >= F || m >= M) return;
        f32x4 a;
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = v[0][i] / (1.f + expf(-v[0][i])) * v[1][i];
        u32x2 hi, lo;
        split_elem4(a, hi, lo);
        *reinterpret_cast<u32x2*>(act + operand_offset(m, n, act_tiles)) = hi;
        *reinterpret_cast<u32x2*>(act + operand_offset(pair_rows + m, n, act_tiles)) = lo;
    }
};

// Fused Q/K/V projection.  A band holds eight channels of one head and, eight columns further on, their rotary
// partners (channel + D/2), so the rotation needs one exchange between two lanes of the wave that owns the band and
// bands are independent of each other.  Q goes to the query buffer as a pair of planes (hi, lo), K (rotated) and V
// into their cache slots (tiled layouts, see k_cache_offset / v_cache_offset).
struct EpiQKV {
    static constexpr const char* NAME = "EpiQKV";
    static constexpr bool NORMALISED_INPUT = true;
    int Hq, Hkv, D, half, bph;  // bph = D/16 bands per head
    int nt;                     // bands per workgroup tile of the launch that uses this epilogue (1 or 2)
    u16* q_out;  // hi plane; the lo plane starts q_plane elements further on
    int ldq;
    size_t q_plane;
    u16* kc;  // this layer: [Hkv] planes of max_seq * D elements in the tiled layouts (k_cache_offset,
    u16* vc;  //             v_cache_offset)
    int max_seq;
    const float* rope_cos;  // [rows][D/2]
    const float* rope_sin;
    RowPlan plan;
    // The device's own prefix length (may be nullptr: no check).  The rows of this pass go to cache slots plan.P ..;
    // if the host's prefix length is not the device's, those slots may hold committed keys and values, so nothing is
    // written to the cache (the pass is flagged DUO_STATUS_PREFIX_MISMATCH by its first kernel and commits nothing).
    const int32_t* dev_prefix_len;
    int cache_ok;  // set by arm()
    struct Pre {
        float cs[2][4], sn[2][4];
    };
    __device__ __forceinline__ void arm() { cache_ok = !dev_prefix_len || *dev_prefix_len == plan.P; }
    // Column c of band (head, j) is channel 8j + c (c < 8) or its rotary partner D/2 + 8j + c - 8.
    __device__ __forceinline__ void prefetch(int tile, int qi, int c, Pre& p) const {
        // no branch around a load (see EpiResidual::prefetch): a band that is not there repeats the first, rows past M
        // re-read row M - 1, and what is not rotated gets the identity afterwards
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int band = tile * nt + (t < nt ? t : 0), head = band / bph;
            const int d = (band - head * bph) * 8 + (c & 7);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = qi * 4 + i;
                const bool rot = m < plan.M && head < Hq + Hkv;
                const int mc = m < plan.M ? m : plan.M - 1;
                const float cs = rope_cos[mc * half + d], sn = rope_sin[mc * half + d];
                p.cs[t][i] = rot ? cs : 1.f;
                p.sn[t][i] = rot ? sn : 0.f;
            }
        }
    }
    // A lane holds rows 4*qi .. +3 of column c; the partner column is eight lanes away (same rows).
    template <int NTT>
    __device__ __forceinline__ void store(int tile, int qi, int c, const f32x4 (&v)[NTT], const Pre& p, bool use_pre) const {
        static_assert(NTT <= 2, "Pre holds the factors of two bands");
        const bool upper = c >= 8;
#pragma unroll
        for (int t = 0; t < NTT; ++t) {
            const int band = tile * NTT + t, head = band / bph;
            const int d = (band - head * bph) * 8 + (c & 7);
            const int ch = upper ? half + d : d;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = qi * 4 + i;
                const float mine = v[t][i];
                const float other = __shfl_xor(mine, 8, 64);  // both lanes of a pair are active together
                if (m >= plan.M) continue;
                if (head < Hq + Hkv) {
                    const float cs = use_pre ? p.cs[t][i] : rope_cos[m * half + d];
                    const float sn = use_pre ? p.sn[t][i] : rope_sin[m * half + d];
                    const float r = upper ? mine * cs + other * sn : mine * cs - other * sn;
                    if (head < Hq) {
                        u16* q = q_out + (size_t)m * ldq + head * D + ch;
                        const u16 r1 = f32_to_elem(r);
                        q[0] = r1;
                        q[q_plane] = f32_to_elem(r - elem_to_f32(r1));
                    } else if (cache_ok) {
                        u16* kp = kc + (size_t)(head - Hq) * max_seq * D;
                        kp[k_cache_offset(D, plan.slot(m), ch)] = f32_to_elem(r);
                    }
                } else if (cache_ok) {
                    u16* vp = vc + (size_t)(head - Hq - Hkv) * max_seq * D;
                    vp[v_cache_offset(D, plan.slot(m), ch)] = f32_to_elem(mine);
                }
            }
        }
    }
    // A lane holds columns c4 .. c4+3 of row m; the partner columns are 32 lanes away (same row).
    template <int NTT>
    __device__ __forceinline__ void store4(int tile, int m, int c4, const f32x4 (&v)[NTT]) const {
        const bool upper = c4 >= 8;
#pragma unroll
        for (int t = 0; t < NTT; ++t) {
            const int band = tile * NTT + t, head = band / bph;
            const int d = (band - head * bph) * 8 + (c4 & 7);
            const int ch = upper ? half + d : d;
            const f32x4 mine = v[t];
            f32x4 other;
#pragma unroll
            for (int i = 0; i < 4; ++i) other[i] = __shfl_xor(mine[i], 32, 64);
            if (m >= plan.M) continue;
            if (head < Hq + Hkv) {
                const f32x4 cs = *reinterpret_cast<const f32x4*>(rope_cos + m * half + d);
                const f32x4 sn = *reinterpret_cast<const f32x4*>(rope_sin + m * half + d);
                const f32x4 r = upper ? mine * cs + other * sn : mine * cs - other * sn;
                if (head < Hq) {
                    u16* q = q_out + (size_t)m * ldq + head * D + ch;
                    u32x2 r1, r2;
                    split_elem4(r, r1, r2);
                    *reinterpret_cast<u32x2*>(q) = r1;
                    *reinterpret_cast<u32x2*>(q + q_plane) = r2;
                } else if (cache_ok) {  // four consecutive channels are contiguous in a key tile
                    u16* kp = kc + (size_t)(head - Hq) * max_seq * D;
                    *reinterpret_cast<u32x2*>(kp + k_cache_offset(D, plan.slot(m), ch)) = pack_elem4(r);
                }
            } else if (cache_ok) {  // the value tiles keep eight SLOTS of one channel together: element stores
                u16* vp = vc + (size_t)(head - Hq - Hkv) * max_seq * D;
#pragma unroll
                for (int i = 0; i < 4; ++i) vp[v_cache_offset(D, plan.slot(m), ch + i)] = f32_to_elem(mine[i]);
            }
        }
    }
};

// Rows of the A operand for M paired activations: hi rows [0, pair_rows), lo rows [pair_rows, 2*pair_rows).
// Up to eight rows share one 16-row tile with their lo halves; beyond that hi and lo halves occupy whole tiles
// (lo tile = hi tile + M/16 rounded up), so a lane's hi and lo sums have the same position in their tiles.
static inline int pair_rows_for(int M) { return M <= 8 ? 8 : (M + 15) / 16 * 16; }
static inline int a_tiles_for(int M, bool paired) { return paired ? (2 * pair_rows_for(M) + 15) / 16 : (M + 15) / 16; }

template <int MT, int NT, int NW, class Epi>
static inline void launch_gemm_cfg(const u16* X, const u16* W, int K, int tiles, int quads, int pq, const RowScale& rsc,
                                   const Epi& epi, hipStream_t s) {
    constexpr int PF = (NT + MT) <= 4 ? 8 : ((NT + MT) <= 8 ? 4 : 2);
    constexpr int GRP = 2;
    DUO_KERNEL_NAME("gemm_skinny_kernel<%d, %d, %d, %d, %d, %s, true>", MT, NT, NW, PF, GRP, Epi::NAME);
    DUO_LAUNCH((gemm_skinny_kernel<MT, NT, NW, PF, GRP, Epi>), dim3(tiles), dim3(NW * 64), s, X, W, K, quads, pq, rsc, epi);
}

// One wave per workgroup when there are enough bands to fill the chip on their own (no partial sums to
// add); otherwise several waves split K.
template <int MT, int NT, class Epi>
static inline void launch_gemm(const u16* X, const u16* W, int K, int tiles, int quads, int pq, const RowScale& rsc,
                               const Epi& epi, hipStream_t s) {
    constexpr int NWK = MT <= 6 ? 4 : 2;  // keeps the partial-sum buffer within 64 KiB of LDS
    if (tiles >= 320) launch_gemm_cfg<MT, NT, 1>(X, W, K, tiles, quads, pq, rsc, epi, s);
    else launch_gemm_cfg<MT, NT, NWK>(X, W, K, tiles, quads, pq, rsc, epi, s);
}

// M output rows; paired: the activations are bf16 pairs (rows m and pair_rows + m of the operand).
template <int NT, class Epi>
static inline void launch_gemm_rows(int M, bool paired, const u16* X, const u16* W, int K, int tiles, const RowScale& rsc,
                                    const Epi& epi, hipStream_t s) {
    const int mt = a_tiles_for(M, paired);
    const int quads = paired ? pair_rows_for(M) / 4 : (M + 3) / 4;
    const int pq = paired ? pair_rows_for(M) / 4 : 0;
    switch (mt) {
        case 1: launch_gemm<1, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
        case 2: launch_gemm<2, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
        case 3: launch_gemm<3, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
        case 4: launch_gemm<4, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
        case 5: launch_gemm<5, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
        case 6: launch_gemm<6, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
        case 7: launch_gemm<7, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
        case 8: launch_gemm<8, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
        case 9: launch_gemm<9, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
        default: launch_gemm<10, NT>(X, W, K, tiles, quads, pq, rsc, epi, s); break;
    }
}

// ---- more than eight rows: the LDS-shared variant ---------------------------------------------------
// Launch shapes measured on the 7B / 8B projections (16..80 rows): 8 weight slots, rounds of 4 K steps, and
// as many consumer waves side by side as keeps the grid just within one workgroup per compute unit.
constexpr int WIDE_MAX_SPLIT = 8;
constexpr int WIDE_PF = 8, WIDE_AG = 4;

template <int MH, int NT, int NG, int NK, class Epi, bool HALF = false, bool STREAM = true>
static inline void launch_wide_cfg(const u16* X, const u16* W, int K, int tiles, int quads, int splits, const RowScale& rsc,
                                   const Epi& epi, hipStream_t s, int* splits_out) {
    // rounds of NK * AG K steps; a round's operand tiles (2*MH per step) must fit the producer's counted wait
    constexpr int AG = (NK * WIDE_AG * (HALF ? 1 : 2 * MH) <= 63) ? WIDE_AG : 2;
    constexpr int RS = NK * AG;
    const int steps = K >> 5;
    int split_steps = (steps + splits - 1) / splits;
    split_steps = (split_steps + RS - 1) / RS * RS;  // whole rounds: only the last split has a ragged end
    const int S = (steps + split_steps - 1) / split_steps;
    if (splits_out) *splits_out = S;
    DUO_KERNEL_NAME("gemm_wide_kernel<%d, %d, %d, %d, %d, %d, %s, %s, %s>", MH, NT, NG, NK, WIDE_PF, AG, Epi::NAME, HALF ? "true" : "false",
                    STREAM ? "true" : "false");
    DUO_LAUNCH((gemm_wide_kernel<MH, NT, NG, NK, WIDE_PF, AG, Epi, HALF, STREAM>), dim3((tiles + NG - 1) / NG, S),
               dim3((NG * NK + 1) * 64), s, X, W, K, split_steps, tiles, quads, rsc, epi);
}

// Projections with many bands (QKV, gate/up, LM head): no K split, the epilogue finishes the rows.
template <int MH, int NT, class Epi>
static inline void launch_wide(const u16* X, const u16* W, int K, int tiles, int quads, const RowScale& rsc, const Epi& epi,
                               hipStream_t s) {
    // few bands: two waves per band group split K, so that four SIMDs per compute unit issue MFMAs
    const int ng = (tiles + 255) / 256;
    if (ng <= 1) launch_wide_cfg<MH, NT, 1, 2>(X, W, K, tiles, quads, 1, rsc, epi, s, nullptr);
    else if (ng == 2) launch_wide_cfg<MH, NT, 2, 2>(X, W, K, tiles, quads, 1, rsc, epi, s, nullptr);
    else if (ng == 3) launch_wide_cfg<MH, NT, 3, 1>(X, W, K, tiles, quads, 1, rsc, epi, s, nullptr);
    else launch_wide_cfg<MH, NT, 4, 1>(X, W, K, tiles, quads, 1, rsc, epi, s, nullptr);
}

// Up to eight rows (hi and lo halves in one operand tile): the same kernel pays for matrices of 257..768 workgroup
// tiles (measured at 4096 input channels: 32.0 against 33.5 us for 688 tiles of two bands, 18.5 against 18.9 us for
// 768 tiles of one band; not for 1000 tiles).  Returns false when the caller should use gemm_skinny_kernel.
template <int NT, class Epi>
static inline bool launch_wide_half(const u16* X, const u16* W, int K, int tiles, const RowScale& rsc, const Epi& epi,
                                    hipStream_t s) {
    if (tiles <= 256 || tiles > 768) return false;
    if (tiles <= 512) launch_wide_cfg<1, NT, 1, 1, Epi, true>(X, W, K, tiles, 2, 1, rsc, epi, s, nullptr);
    else launch_wide_cfg<1, NT, 3, 1, Epi, true>(X, W, K, tiles, 2, 1, rsc, epi, s, nullptr);
    return true;
}

// Projections with few bands (O, down): K is split over the grid's y dimension and the workgroups store
// partial results [split][M][N]; residual_reduce_kernel adds them in split order.  Returns the number of splits.
template <int MH>
static inline int launch_wide_split(const u16* X, const u16* W, int K, int N, int M, float* part, const RowScale& rsc,
                                    hipStream_t s) {
    EpiStoreF32 e{N, M, 1, part, N, (size_t)M * N};
    const int quads = pair_rows_for(M) / 4;
    int S = 1;
    // eight splits of eight-band workgroups, also for the shorter K of the O projection (measured at 64 rows, 4096 x 4096:
    // 11.7 against 12.2 us for four splits of four-band workgroups)
    launch_wide_cfg<MH, 1, 8, 1>(X, W, K, N / 16, quads, WIDE_MAX_SPLIT, rsc, e, s, &S);
    return S;
}
