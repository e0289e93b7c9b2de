// Speculative sampling over the target logits (Alg. 2, Sec. 3.3) and the KV commit.
//
// All probabilities are evaluated in double from the fp32 logits, so that the accept decision
// u * q(t) < p(t) and the inverse-CDF draws are taken in the precision a plain reference uses;
// the volumes are tiny next to the weight stream (two passes over a few vocabulary rows).
//   sample_stats_kernel   max and normaliser of softmax(logits / T) for every row of logits, the vocabulary cut into
//                         slices for parallelism (caller-supplied logits only: in the verify step the LM head's
//                         epilogue leaves these statistics, one part per 32-column tile, see EpiLogitsStats)
//   sample_finish_kernel  one workgroup per sequence: accept flags, leading accepts, then the
//                         correction token from norm(max(0, p - q)) or the bonus token from p
//   sample_row_stats_kernel, sample_spread_kernel, sample_locate_kernel
//                         the same rule for vocabularies of SPREAD_MIN_VOCAB entries and more, spread over many
//                         workgroups (see there)
//   sample_paper_kernel   the sequential first-token rule over the n sequences, with the
//                         running distribution replaced by its residual after each rejection
//   sample_deferred_kernel  Alg. 2 as listed: verify the unverified suffix, then judge only the first
//                         tokens of the new sequences
//   commit_kernel         picks the sequence to keep, moves its accepted K/V next to the prefix
//
// T = 0 is the greedy limit of the same rule: softmax(logits / T) tends to the one-hot distribution at the
// largest logit (lowest id among equals), so a draft token is accepted exactly when it is that id, and every
// correction or bonus token is that id (p(t) in {0, 1} in u * q(t) < p(t); the residual of a one-hot p is the
// same one-hot unless q already puts all its mass there).  The statistics then hold the arg max instead of the
// normaliser; everything else runs unchanged on the one-hot p.
//
// Nucleus (top-p) restriction of the target distributions: sample_nucleus_kernel finds, per judging row, the
// set of most probable tokens whose mass reaches top_p (equal probabilities by ascending id) as a threshold on
// the logit plus the last admitted id among the logits equal to it, and the kept mass; the kernels above then
// evaluate p'(v) = p(v) / kept mass inside the set and 0 outside.  Without it (nuc == nullptr) nothing changes.
#pragma once
#include "duo_common.h"

struct SampleArgs {
    const float* logits;  // fp32 [R + n*k][ld]
    int ld;
    const float* root_logits;  // fp32 [V], judges first tokens when R == 0
    int V, n, k, R, P;
    double T;               // temperature; 0 selects the greedy limit
    const int32_t* tokens;  // [n][k]
    const float* q;         // [n][k][V]
    const float* u;         // [n][k+1]
    // Softmax statistics of the judging rows, as partial results over slices of the vocabulary: per slice the max of
    // z = logit / T and sum exp(z - max) (greedy: the max logit and the lowest id that attains it).  stats_rows
    // [R + n*k][parts][2] belongs to the rows of `logits`: written by the LM head's epilogue (one part per 32-column
    // tile) or by sample_stats_kernel (STATS_SPLIT parts); stats_root [root_parts][2] to root_logits (R == 0).
    double* stats_rows;
    int parts;
    double* stats_root;
    int root_parts;  // STATS_SPLIT from sample_stats_kernel, ROOT_STATS_PARTS from the verify pass's first kernel
    int32_t* acc;           // [n][k] accept flags
    double* p_run;          // [V] running distribution of the sequential rule
    int32_t* accept_len;    // [n]
    int32_t* next_token;    // [n]
    int32_t* commit;        // [4]
    int32_t* status;
    const double* nuc;      // nucleus records [1 + n*k][4] (threshold key, last tied id, kept mass, -), or nullptr
    __device__ __forceinline__ int nuc_row(int i, int j) const { return j == 0 ? 0 : 1 + i * k + (j - 1); }
    // row of `logits` that judges draft (i, j), or -1 for root_logits
    __device__ __forceinline__ int judge_index(int i, int j) const { return j == 0 ? (R ? 0 : -1) : R + i * k + j - 1; }
    __device__ __forceinline__ const float* judge_row(int i, int j) const {
        if (j == 0) return R ? logits : root_logits;
        return logits + (size_t)(R + i * k + j - 1) * ld;
    }
    __device__ __forceinline__ bool greedy() const { return T == 0.0; }
    __device__ __forceinline__ int token(int i, int j) const {
        int t = tokens[i * k + j];
        return t < 0 ? 0 : (t >= V ? V - 1 : t);
    }
};

// The status word as the kernels before this one left it (they OR their flags in with device-scope atomics).  A pass
// whose status is not clean commits nothing: the device prefix length and every cache slot below it stay as they
// were, and the commit record reads {-1, 0, -1, unchanged prefix length}.
__device__ __forceinline__ int32_t status_now(int32_t* status) {
    return status ? __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
}
// commit record of a pass that failed on the device; P is the host's prefix length, used when there is no cache
__device__ __forceinline__ void write_failed_commit(int32_t* commit, const int32_t* prefix_len, int P) {
    commit[0] = -1;
    commit[1] = 0;
    commit[2] = -1;
    commit[3] = prefix_len ? *prefix_len : P;
}

// Logits as unsigned keys in the same order (-0 counted as +0), and the nucleus test of one token.
__device__ __forceinline__ uint32_t logit_key(float x) {
    const uint32_t b = __float_as_uint(x + 0.0f);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
struct Nucleus {
    bool on;
    uint32_t thr;  // kept: key > thr, or key == thr and id <= vcut
    int vcut;
    double inv;    // 1 / kept mass
    __device__ __forceinline__ bool keeps(float logit, int v) const {
        const uint32_t kx = logit_key(logit);
        return kx > thr || (kx == thr && v <= vcut);
    }
    // p (already normalised over the whole vocabulary) -> p'
    __device__ __forceinline__ double apply(double p, float logit, int v) const {
        return !on ? p : (keeps(logit, v) ? p * inv : 0.0);
    }
};
// NUC = false: the kernels are compiled without the restriction (nothing of it is left in their loops)
template <bool NUC>
__device__ __forceinline__ Nucleus nucleus_of(const SampleArgs& a, int i, int j) {
    if (!NUC || !a.nuc) return Nucleus{false, 0u, 0, 1.0};
    const double* e = a.nuc + (size_t)a.nuc_row(i, j) * 4;
    return Nucleus{true, (uint32_t)e[0], (int)e[1], 1.0 / e[2]};
}

constexpr int SAMPLE_THREADS = 1024;
constexpr int STATS_SPLIT = 8;        // workgroups per row of logits in sample_stats_kernel
constexpr int ROOT_STATS_PARTS = 32;  // slices of the cached root logits when the verify pass's first kernel takes their statistics

__device__ __forceinline__ double block_sum_d(double v, double* sm) {
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    __syncthreads();
    if (lane == 0) sm[wave] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < nw; ++w) t += sm[w];
    return t;
}
__device__ __forceinline__ double block_max_d(double v, double* sm) {
    v = wave_max(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    __syncthreads();
    if (lane == 0) sm[wave] = v;
    __syncthreads();
    double t = sm[0];
    for (int w = 1; w < nw; ++w) t = fmax(t, sm[w]);
    return t;
}

// Statistics of one slice [v0, v1) of a row of logits (all 256 threads of the workgroup): zmax and Z as SampleArgs
// describes them.
__device__ __forceinline__ void slice_stats(const float* __restrict__ row, int v0, int v1, double T, double* sm, double& zmax,
                                            double& Z) {
    float lm = -INFINITY;
    for (int v = v0 + threadIdx.x; v < v1; v += 256) lm = fmaxf(lm, row[v]);
    if (T == 0.0) {  // Z: the lowest id of the slice that holds the slice's largest logit
        zmax = block_max_d((double)lm, sm);
        int first = 0x7fffffff;
        for (int v = v0 + threadIdx.x; v < v1; v += 256)
            if ((double)row[v] == zmax) first = min(first, v);
        Z = -block_max_d(-(double)first, sm);
    } else {
        zmax = block_max_d((double)lm, sm) / T;
        double s = 0.0;
        for (int v = v0 + threadIdx.x; v < v1; v += 256) s += exp((double)row[v] / T - zmax);
        Z = block_sum_d(s, sm);
    }
}

// grid (R + n*k + (R ? 0 : 1), STATS_SPLIT): slice sl of row r of `logits`, the last row index being root_logits when
// there is no root row.  Used when the logits come from the caller; the verify step's LM head leaves the same
// statistics itself (EpiLogitsStats in duo_gemm.h) and the pass's first kernel those of root_logits.
__global__ __launch_bounds__(256) void sample_stats_kernel(SampleArgs a) {
    __shared__ double sm[16];
    const int r = blockIdx.x, sl = blockIdx.y, rows = a.R + a.n * a.k;
    const float* row = r < rows ? a.logits + (size_t)r * a.ld : a.root_logits;
    const int len = (a.V + STATS_SPLIT - 1) / STATS_SPLIT;
    const int v0 = sl * len, v1 = min(a.V, v0 + len);
    double zmax, Z;
    slice_stats(row, v0, v1, a.T, sm, zmax, Z);
    if (threadIdx.x == 0) {
        double* st = (r < rows ? a.stats_rows + ((size_t)r * a.parts + sl) * 2 : a.stats_root + sl * 2);
        st[0] = zmax;
        st[1] = Z;
        const int t = r - a.R;  // the draft token this row belongs to
        if (sl == 0 && t >= 0 && t < a.n * a.k) {
            const int raw = a.tokens[t];
            if ((raw < 0 || raw >= a.V) && a.status) atomicOr(a.status, 1);
        }
    }
}

// The merged statistics of the judging rows of one sequence, position j -> {zmax, Z} (greedy: {max logit, arg max}),
// kept in shared memory by the kernels below.
struct SeqStats {
    double (*t)[2];
};

// Merge of the partial statistics of judging rows (i, j0 .. j1) into st.t[j]: one wave per row, lanes stride over the
// parts, fixed butterflies (deterministic).  All threads of the workgroup call it; ends with a barrier.
__device__ __forceinline__ void load_seq_stats(const SampleArgs& a, int i, int j0, int j1, const SeqStats& st) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    for (int j = j0 + wave; j <= j1; j += nw) {
        const int jr = a.judge_index(i, j);
        const double* pt = jr < 0 ? a.stats_root : a.stats_rows + (size_t)jr * a.parts * 2;
        const int np = jr < 0 ? a.root_parts : a.parts;
        double mx = -INFINITY;
#pragma unroll 4
        for (int p = lane; p < np; p += 64) mx = fmax(mx, pt[2 * p]);
        mx = wave_max(mx);
        double Z;
        if (a.greedy()) {  // the lowest id among the parts that hold the largest logit (parts are in id order)
            double first = 4.0e9;
            for (int p = lane; p < np; p += 64)
                if (pt[2 * p] == mx) first = fmin(first, pt[2 * p + 1]);
            Z = -wave_max(-first);
        } else {
            double sum = 0.0;
#pragma unroll 4
            for (int p = lane; p < np; p += 64)
                if (pt[2 * p + 1] > 0.0) sum += pt[2 * p + 1] * exp(pt[2 * p] - mx);
            Z = wave_sum(sum);
        }
        if (lane == 0) {
            st.t[j][0] = mx;
            st.t[j][1] = Z;
        }
    }
    __syncthreads();
}

__device__ __forceinline__ void merged_stats(const SeqStats& st, int j, double& zmax, double& Z) {
    zmax = st.t[j][0];
    Z = st.t[j][1];
}
__device__ __forceinline__ int merged_argmax(const SeqStats& st, int j) { return (int)st.t[j][1]; }

// p_run[v] = p(v) of judging distribution (i, j) for the whole vocabulary; ends with a barrier
template <bool NUC>
__device__ __forceinline__ void fill_running_distribution(const SampleArgs& a, const SeqStats& st, int i, int j) {
    const float* row = a.judge_row(i, j);
    if (a.greedy()) {
        const int amax = merged_argmax(st, j);
        for (int v = threadIdx.x; v < a.V; v += blockDim.x) a.p_run[v] = v == amax ? 1.0 : 0.0;
    } else {
        double zmax, Z;
        merged_stats(st, j, zmax, Z);
        const Nucleus nc = nucleus_of<NUC>(a, i, j);
        for (int v = threadIdx.x; v < a.V; v += blockDim.x)
            a.p_run[v] = nc.apply(exp((double)row[v] / a.T - zmax) / Z, row[v], v);
    }
    __syncthreads();
}

// One workgroup per judging row r (0 = the root distribution, 1 + i*k + (j-1) = row (i, j)).  `prow` ([rows][V]
// doubles) holds the row's probabilities while the threshold is searched: bit by bit from the top, the largest
// logit key t with mass{key >= t} >= top_p * total (32 block sums in a fixed order), then as many of the ids that
// sit exactly on the threshold, in ascending order, as the target still needs.
// PT > 0: the vocabulary has at most PT * 1024 entries and every thread keeps its PT keys and probabilities in
// registers for the 33 passes (they are latency-bound otherwise: 340 -> 120 us for nine rows of 32000); PT = 0: any
// vocabulary, the passes re-read the row.
template <int PT>
__global__ __launch_bounds__(SAMPLE_THREADS) void sample_nucleus_kernel(SampleArgs a, double top_p, double* __restrict__ prow_all,
                                                                        double* __restrict__ nuc_out) {
    __shared__ double sm_d[16];
    __shared__ int sm_i[SAMPLE_THREADS / 64 + 2];
    __shared__ double sm_st[DUO_MAX_ROWS + 1][2];
    const SeqStats st{sm_st};
    const int r = blockIdx.x, tid = threadIdx.x;
    const int i = r == 0 ? 0 : (r - 1) / a.k, j = r == 0 ? 0 : (r - 1) % a.k + 1;
    const float* row = a.judge_row(i, j);
    double* prow = prow_all + (size_t)r * a.V;
    load_seq_stats(a, i, j, j, st);
    double zmax, Z;
    merged_stats(st, j, zmax, Z);
    constexpr int NR = PT > 0 ? PT : 1;
    uint32_t rk[NR];  // PT > 0: this thread's keys and probabilities, ids tid + e * 1024 (beyond the vocabulary: none)
    double rp[NR];
    double loc = 0.0;
    if (PT > 0) {
#pragma unroll
        for (int e = 0; e < NR; ++e) {
            const int v = tid + e * SAMPLE_THREADS;
            const bool in = v < a.V;
            const float x = row[in ? v : 0];
            const double p = in ? exp((double)x / a.T - zmax) / Z : 0.0;
            rk[e] = in ? logit_key(x) : 0u;
            rp[e] = p;
            if (in) prow[v] = p;
            loc += p;
        }
    } else {
        for (int v = tid; v < a.V; v += SAMPLE_THREADS) {
            const double p = exp((double)row[v] / a.T - zmax) / Z;
            prow[v] = p;
            loc += p;
        }
    }
    const double target = top_p * block_sum_d(loc, sm_d);  // also orders the prow writes before the reads below
    auto mass_from = [&](uint32_t t, bool strictly) {  // mass of the keys >= t (or > t); same order of additions either way
        double s = 0.0;
        if (PT > 0) {
#pragma unroll
            for (int e = 0; e < NR; ++e) s += (strictly ? rk[e] > t : rk[e] >= t) ? rp[e] : 0.0;
        } else {
            for (int v = tid; v < a.V; v += SAMPLE_THREADS) {
                const uint32_t kx = logit_key(row[v]);
                s += (strictly ? kx > t : kx >= t) ? prow[v] : 0.0;
            }
        }
        return block_sum_d(s, sm_d);
    };
    uint32_t cur = 0u;
    for (int b = 31; b >= 0; --b) {
        const uint32_t t = cur | (1u << b);
        if (mass_from(t, false) >= target) cur = t;  // same value in every thread
    }
    const double above = mass_from(cur, true);
    // the ids on the threshold share one probability; ids in ascending order: contiguous ranges per thread
    const int per = (a.V + SAMPLE_THREADS - 1) / SAMPLE_THREADS;
    const int v0 = min(a.V, tid * per), v1 = min(a.V, v0 + per);
    int cnt = 0;
    double pstar = 0.0;
    for (int v = v0; v < v1; ++v)
        if (logit_key(row[v]) == cur) {
            ++cnt;
            pstar = prow[v];
        }
    pstar = block_max_d(pstar, sm_d);
    int need = (int)ceil((target - above) / pstar);
    need = need < 1 ? 1 : need;
    while (need > 1 && above + (double)(need - 1) * pstar >= target) --need;
    while (above + (double)need * pstar < target) ++need;
    // exclusive scan of the per-thread counts (lanes, then waves in index order)
    const int lane = tid & 63, wave = tid >> 6;
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o, 64);
        if (lane >= o) incl += y;
    }
    __syncthreads();
    if (lane == 63) sm_i[wave] = incl;
    if (tid == 0) sm_i[SAMPLE_THREADS / 64] = a.V - 1;
    __syncthreads();
    int before = incl - cnt, total_ties = 0;
    for (int w = 0; w < SAMPLE_THREADS / 64; ++w) {
        if (w < wave) before += sm_i[w];
        total_ties += sm_i[w];
    }
    need = need > total_ties ? total_ties : need;  // rounding asked for more than there are: all of them
    if (cnt > 0 && before < need && need <= before + cnt) {  // the need-th tied id lies in this thread's range
        int seen = before;
        for (int v = v0; v < v1; ++v)
            if (logit_key(row[v]) == cur && ++seen == need) sm_i[SAMPLE_THREADS / 64] = v;
    }
    __syncthreads();
    if (tid == 0) {
        double* e = nuc_out + (size_t)r * 4;
        e[0] = (double)cur;
        e[1] = (double)sm_i[SAMPLE_THREADS / 64];
        e[2] = above + (double)need * pstar;
        e[3] = (double)need;
    }
}

// accept flags of sequence i, positions from..k-1 (one thread each), into acc[]; ends with a barrier
// the accept test u * q(t) < p(t) of draft (i, j)
template <bool NUC>
__device__ __forceinline__ int accept_flag(const SampleArgs& a, const SeqStats& st, int i, int j) {
    const float* row = a.judge_row(i, j);
    const int t = a.token(i, j);
    double p_t;
    if (a.greedy()) {
        p_t = t == merged_argmax(st, j) ? 1.0 : 0.0;
    } else {
        double zmax, Z;
        merged_stats(st, j, zmax, Z);
        p_t = nucleus_of<NUC>(a, i, j).apply(exp((double)row[t] / a.T - zmax) / Z, row[t], t);
    }
    const double lhs = (double)a.u[i * (a.k + 1) + j] * (double)a.q[((size_t)i * a.k + j) * a.V + t];
    return lhs < p_t ? 1 : 0;
}
template <bool NUC>
__device__ __forceinline__ void accept_flags(const SampleArgs& a, const SeqStats& st, int i, int from) {
    const int j = from + threadIdx.x;
    if (j < a.k) a.acc[i * a.k + j] = accept_flag<NUC>(a, st, i, j);
    __threadfence_block();
    __syncthreads();
}

// Inverse CDF over non-negative weights w(v), v ascending: smallest v whose running sum exceeds
// u * total.  Every wave owns a contiguous chunk of the vocabulary and reads it 64 consecutive ids at a
// time (coalesced; the loads of a chunk do not depend on each other).  First the chunk sums, added over
// the waves in index order, locate the chunk where the running sum crosses the target; then that wave
// alone narrows it down (lane segments, then a scan inside the crossing segment).
// Returns (to every thread) the token, or -1 if the total is zero.
template <class F>
__device__ int block_inverse_cdf(F w, int V, double u, double* sm_d, int* sm_i) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, nw = blockDim.x >> 6;
    const int chunk = ((V + nw - 1) / nw + 63) / 64 * 64;
    const int c0 = wave * chunk, c1 = min(V, c0 + chunk);
    double local = 0.0;
    int lastpos = -1;
#pragma unroll 4
    for (int v = c0 + lane; v < c1; v += 64) {
        const double x = w(v);
        local += x;
        if (x > 0.0) lastpos = v;
    }
    const double csum = wave_sum(local);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lastpos = max(lastpos, __shfl_xor(lastpos, o, 64));
    __syncthreads();
    if (lane == 0) {
        sm_d[wave] = csum;
        sm_i[4 + wave] = lastpos;
    }
    __syncthreads();
    double total = 0.0;
    for (int ww = 0; ww < nw; ++ww) total += sm_d[ww];
    if (!(total > 0.0)) return -1;
    const double target = u * total;
    // the first chunk whose inclusive sum exceeds the target, and the running sum before it
    int owner = -1, last_all = -1;
    double base = 0.0, run = 0.0;
    for (int ww = 0; ww < nw; ++ww) {
        if (owner < 0 && run + sm_d[ww] > target) {
            owner = ww;
            base = run;
        }
        run += sm_d[ww];
        last_all = max(last_all, sm_i[4 + ww]);
    }
    if (owner < 0) return last_all;  // rounding left no crossing: largest id with positive weight
    if (wave == owner) {
        // Lane l re-adds ids [c0 + l*per, +per) of the chunk; a scan over the lanes finds the lane whose
        // segment holds the crossing; the wave then walks that segment 64 ids at a time.
        const int per = chunk >> 6;
        const int s0 = c0 + lane * per, s1 = min(c1, s0 + per);
        double seg = 0.0;
#pragma unroll 4
        for (int v = s0; v < s1; ++v) seg += w(v);
        double incl = seg;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double y = __shfl_up(incl, o, 64);
            if (lane >= o) incl += y;
        }
        const unsigned long long hit = __ballot(base + incl > target);
        int tok = -1;
        if (hit) {
            const int hl = __ffsll((long long)hit) - 1;
            double before = base + __shfl(incl - seg, hl, 64);  // running sum in front of that segment
            const int h0 = c0 + hl * per, h1 = min(c1, h0 + per);
            for (int v0 = h0; v0 < h1 && tok < 0; v0 += 64) {
                const int v = v0 + lane;
                const double x = v < h1 ? w(v) : 0.0;
                double ix = x;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const double y = __shfl_up(ix, o, 64);
                    if (lane >= o) ix += y;
                }
                const unsigned long long h2 = __ballot(before + ix > target);
                if (h2) tok = v0 + __ffsll((long long)h2) - 1;
                before += __shfl(ix, 63, 64);
            }
        }
        // the chunk sum crossed but, in this summation order, no prefix did: its last positive id
        if (lane == 0) sm_i[2] = tok >= 0 ? tok : sm_i[4 + wave];
    }
    __syncthreads();
    return sm_i[2];
}

// Correction / bonus token of sequence i after `a` accepted drafts.
template <bool NUC>
__device__ int finish_token(const SampleArgs& a, const SeqStats& st, int i, int acc_len, double* sm_d, int* sm_i) {
    const float* row = a.judge_row(i, acc_len);
    if (a.greedy()) {  // one-hot p: same two draws over the one-hot weights
        const int amax = merged_argmax(st, acc_len);
        const double ug = (double)a.u[i * (a.k + 1) + a.k];
        auto pg = [=](int v) { return v == amax ? 1.0 : 0.0; };
        if (acc_len < a.k) {
            const float* qrow = a.q + ((size_t)i * a.k + acc_len) * a.V;
            auto rg = [=](int v) { return fmax((v == amax ? 1.0 : 0.0) - (double)qrow[v], 0.0); };
            const int tok = block_inverse_cdf(rg, a.V, ug, sm_d, sm_i);
            if (tok >= 0) return tok;
        }
        return block_inverse_cdf(pg, a.V, ug, sm_d, sm_i);
    }
    double zmax, Z;
    merged_stats(st, acc_len, zmax, Z);
    // reciprocals once per call instead of two divisions per vocabulary entry (the single workgroup is
    // bound by its double-precision arithmetic); the results differ from the quotients by an ulp at most
    const double iT = 1.0 / a.T, iZ = 1.0 / Z;
    const double u = (double)a.u[i * (a.k + 1) + a.k];
    const Nucleus nc = nucleus_of<NUC>(a, i, acc_len);
    auto pw = [=](int v) { return nc.apply(exp((double)row[v] * iT - zmax) * iZ, row[v], v); };
    if (acc_len < a.k) {
        const float* qrow = a.q + ((size_t)i * a.k + acc_len) * a.V;
        auto rw = [=](int v) { return fmax(nc.apply(exp((double)row[v] * iT - zmax) * iZ, row[v], v) - (double)qrow[v], 0.0); };
        const int tok = block_inverse_cdf(rw, a.V, u, sm_d, sm_i);
        if (tok >= 0) return tok;  // else: the residual vanished (p == q), fall back to p
    }
    return block_inverse_cdf(pw, a.V, u, sm_d, sm_i);
}

__device__ __forceinline__ int leading_accepts(const SampleArgs& a, int i, int from) {
    int n = from;
    while (n < a.k && a.acc[i * a.k + n]) ++n;
    return n;
}

// self_commit (single-sequence calls): also write the commit record and advance the device prefix length, which
// otherwise commit_kernel does after choosing among the sequences.
template <bool NUC>
__global__ __launch_bounds__(SAMPLE_THREADS) void sample_finish_kernel(SampleArgs a, int self_commit, int32_t* prefix_len) {
    __shared__ double sm_d[16];
    __shared__ int sm_i[4 + 16];
    __shared__ double sm_st[DUO_MAX_ROWS + 1][2];
    const SeqStats st{sm_st};
    const int i = blockIdx.x;
    load_seq_stats(a, i, 0, a.k, st);
    accept_flags<NUC>(a, st, i, 0);
    const int acc_len = leading_accepts(a, i, 0);
    const int tok = finish_token<NUC>(a, st, i, acc_len, sm_d, sm_i);
    if (threadIdx.x == 0) {
        a.accept_len[i] = acc_len;
        a.next_token[i] = tok;
        if (self_commit) {
            if (status_now(a.status) != 0) {
                write_failed_commit(a.commit, prefix_len, a.P);
            } else {
                a.commit[0] = 0;
                a.commit[1] = acc_len;
                a.commit[2] = tok;
                a.commit[3] = a.P + a.R + acc_len;
                if (prefix_len) *prefix_len = a.P + a.R + acc_len;
            }
        }
    }
}

// ---- the same rule for large vocabularies, spread over the chip ----------------------------------------------
// sample_finish_kernel is one workgroup per sequence and bound by its double-precision arithmetic: the merge of the
// rows' partial statistics (vocab / 32 parts per row after the LM head) and the pass over the vocabulary behind the
// correction token each evaluate tens of thousands of exponentials on one compute unit (27 us at 32000 entries, 87 us at
// 128256).  Three small kernels do the same work on many:
//   sample_row_stats_kernel   one workgroup per judging row: its merged statistics {zmax, Z}
//   sample_spread_kernel      grid (sequence, slice of the vocabulary): accept flags and leading accepts (every slice
//                             repeats them: k exponentials), then the sums of the correction weights max(0, p - q)
//                             and of p over the slice's 16 wave chunks, with the last id of positive weight in each
//   sample_locate_kernel      one wave per sequence: the chunk in which the running sum crosses u * total (chunk sums
//                             added in index order), the id inside it, the commit record of a single sequence
// Their scratch (SpreadBuf) lies in p_run, which this rule does not use otherwise.
struct SpreadBuf {
    double* row_stats;  // [R + n*k + 1][2], row judge_index + 1
    double* sums;       // [n][chunks][2]: correction weights, target probabilities
    int32_t* last;      // [n][chunks][2]
    int G, chunk;       // slices per sequence; ids per wave chunk (a multiple of 64); chunks = 16 * G
    __host__ __device__ int chunks() const { return 16 * G; }
};
constexpr int SPREAD_MIN_VOCAB = 8192;   // below: sample_finish_kernel
constexpr int SPREAD_MAX_GROUPS = 128;   // n * G at most: the records fit SPREAD_MIN_VOCAB doubles
constexpr int SPREAD_MAX_SLICES = 32;

__global__ __launch_bounds__(256) void sample_row_stats_kernel(SampleArgs a, SpreadBuf b) {
    __shared__ double sm[16];
    const int jr = (int)blockIdx.x - 1;
    if (jr < 0 && a.R) return;  // a root row judges the first tokens: the cached root logits are not in play
    const double* pt = jr < 0 ? a.stats_root : a.stats_rows + (size_t)jr * a.parts * 2;
    const int np = jr < 0 ? a.root_parts : a.parts;
    // a thread's parts stay in registers between the two passes, all of their loads in flight together (up to
    // 256 * PER parts, i.e. a vocabulary of 131072 behind the LM head; more: the passes re-read them)
    constexpr int PER = 16;
    const bool in_regs = np <= 256 * PER;
    double pm[PER], pz[PER];
    if (in_regs) {
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const int p = threadIdx.x + 256 * e;
            const int pc = p < np ? p : np - 1;
            pm[e] = pt[2 * pc];
            pz[e] = pt[2 * pc + 1];
            if (p >= np) {
                pm[e] = -INFINITY;
                pz[e] = 0.0;
            }
        }
    }
    double mx = -INFINITY;
    if (in_regs) {
#pragma unroll
        for (int e = 0; e < PER; ++e) mx = fmax(mx, pm[e]);
    } else {
#pragma unroll 4
        for (int p = threadIdx.x; p < np; p += 256) mx = fmax(mx, pt[2 * p]);
    }
    mx = block_max_d(mx, sm);
    double Z;
    if (a.greedy()) {  // the lowest id among the parts that hold the largest logit
        double first = 4.0e9;
        if (in_regs) {
#pragma unroll
            for (int e = 0; e < PER; ++e)
                if (pm[e] == mx) first = fmin(first, pz[e]);
        } else {
            for (int p = threadIdx.x; p < np; p += 256)
                if (pt[2 * p] == mx) first = fmin(first, pt[2 * p + 1]);
        }
        Z = -block_max_d(-first, sm);
    } else {
        double sum = 0.0;
        if (in_regs) {
#pragma unroll
            for (int e = 0; e < PER; ++e)
                if (pz[e] > 0.0) sum += pz[e] * exp(pm[e] - mx);
        } else {
#pragma unroll 4
            for (int p = threadIdx.x; p < np; p += 256)
                if (pt[2 * p + 1] > 0.0) sum += pt[2 * p + 1] * exp(pt[2 * p] - mx);
        }
        Z = block_sum_d(sum, sm);
    }
    if (threadIdx.x == 0) {
        b.row_stats[2 * blockIdx.x] = mx;
        b.row_stats[2 * blockIdx.x + 1] = Z;
    }
}

// p(v) of judging row (i, j) and the correction weight max(0, p(v) - q(v)) behind a rejection at j < k
template <bool NUC>
struct TokenWeights {
    const float* row;
    const float* qrow;  // nullptr: no draft distribution at this position (bonus token)
    double iT, zmax, iZ;
    int amax;  // greedy: the one-hot id; -1 otherwise
    Nucleus nc;
    // row_zmax, row_Z: the row's merged statistics (greedy: row_Z is the arg max)
    __device__ __forceinline__ TokenWeights(const SampleArgs& a, int i, int j, double row_zmax, double row_Z) {
        row = a.judge_row(i, j);
        qrow = j < a.k ? a.q + ((size_t)i * a.k + j) * a.V : nullptr;
        amax = a.greedy() ? (int)row_Z : -1;
        iT = a.greedy() ? 0.0 : 1.0 / a.T;  // reciprocals once instead of two divisions per entry (an ulp at most)
        zmax = row_zmax;
        iZ = a.greedy() ? 0.0 : 1.0 / row_Z;
        nc = nucleus_of<NUC>(a, i, j);
    }
    __device__ __forceinline__ double p(int v) const {
        if (amax >= 0) return v == amax ? 1.0 : 0.0;
        return nc.apply(exp((double)row[v] * iT - zmax) * iZ, row[v], v);
    }
    __device__ __forceinline__ double r(double pv, int v) const { return fmax(pv - (double)qrow[v], 0.0); }
};

template <bool NUC>
__global__ __launch_bounds__(SAMPLE_THREADS) void sample_spread_kernel(SampleArgs a, SpreadBuf b) {
    __shared__ double sm_st[DUO_MAX_ROWS + 1][2];
    __shared__ int sm_acc[DUO_MAX_ROWS];
    const SeqStats st{sm_st};
    const int i = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (tid <= a.k) {
        const double* rs = b.row_stats + 2 * (a.judge_index(i, tid) + 1);
        sm_st[tid][0] = rs[0];
        sm_st[tid][1] = rs[1];
    }
    __syncthreads();
    if (tid < a.k) sm_acc[tid] = accept_flag<NUC>(a, st, i, tid);
    __syncthreads();
    int acc_len = 0;
    while (acc_len < a.k && sm_acc[acc_len]) ++acc_len;
    if (g == 0 && tid == 0) a.accept_len[i] = acc_len;
    const TokenWeights<NUC> w(a, i, acc_len, sm_st[acc_len][0], sm_st[acc_len][1]);
    const int c = g * 16 + wave;
    const int c0 = min(a.V, c * b.chunk), c1 = min(a.V, c0 + b.chunk);
    double sum_r = 0.0, sum_p = 0.0;
    int last_r = -1, last_p = -1;
    if (w.qrow) {
#pragma unroll 4
        for (int v = c0 + lane; v < c1; v += 64) {
            const double pv = w.p(v), rv = w.r(pv, v);
            sum_p += pv;
            sum_r += rv;
            if (pv > 0.0) last_p = v;
            if (rv > 0.0) last_r = v;
        }
    } else {
#pragma unroll 4
        for (int v = c0 + lane; v < c1; v += 64) {
            const double pv = w.p(v);
            sum_p += pv;
            if (pv > 0.0) last_p = v;
        }
    }
    sum_r = wave_sum(sum_r);
    sum_p = wave_sum(sum_p);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        last_r = max(last_r, __shfl_xor(last_r, o, 64));
        last_p = max(last_p, __shfl_xor(last_p, o, 64));
    }
    if (lane == 0) {
        const size_t e = ((size_t)i * b.chunks() + c) * 2;
        b.sums[e] = sum_r;
        b.sums[e + 1] = sum_p;
        b.last[e] = last_r;
        b.last[e + 1] = last_p;
    }
}

// One wave.  Inverse CDF over the weights whose chunk sums (x[g]: chunk 64 * g + lane, zero beyond the last chunk) and
// last ids of positive weight (lp[g], -1 for none) were left by sample_spread_kernel: smallest id whose running sum
// (chunks in index order, then lane segments of the crossing chunk, then single ids) exceeds u * total; the largest id
// of positive weight where rounding leaves no crossing; -1 if the total is zero.
constexpr int SPREAD_GROUPS64 = SPREAD_MAX_SLICES * 16 / 64;
template <class F>
__device__ int wave_inverse_cdf(F w, int V, double u, const double (&x)[SPREAD_GROUPS64], const int (&lp)[SPREAD_GROUPS64], int chunks,
                                int chunk) {
    const int lane = threadIdx.x & 63;
    // Running sums over the chunks, 64 at a time: an inclusive scan over the lanes on top of the sum of the groups in
    // front.  The total is the last running sum of the same arithmetic, so the search ends on it.
    double incl[SPREAD_GROUPS64], front[SPREAD_GROUPS64], total = 0.0;
    int last_all = -1;
#pragma unroll
    for (int g = 0; g < SPREAD_GROUPS64; ++g) {
        incl[g] = x[g];
        front[g] = total;
        if (g * 64 >= chunks) continue;  // wave-uniform: no chunk in this group
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double y = __shfl_up(incl[g], o, 64);
            if (lane >= o) incl[g] += y;
        }
        total += __shfl(incl[g], 63, 64);
        int l = lp[g];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) l = max(l, __shfl_xor(l, o, 64));
        last_all = max(last_all, l);
    }
    if (!(total > 0.0)) return -1;
    const double target = u * total;
    int owner = -1, owner_last = -1;
    double base = 0.0;
#pragma unroll
    for (int g = 0; g < SPREAD_GROUPS64; ++g) {
        const unsigned long long hit = __ballot(x[g] > 0.0 && front[g] + incl[g] > target);
        if (owner < 0 && hit) {
            const int hl = __ffsll((long long)hit) - 1;
            owner = g * 64 + hl;
            base = front[g] + __shfl(incl[g] - x[g], hl, 64);  // running sum in front of that chunk
            owner_last = __shfl(lp[g], hl, 64);
        }
    }
    if (owner < 0) return last_all;
    const int c0 = min(V, owner * chunk), c1 = min(V, c0 + chunk);
    const int per = chunk >> 6;
    const int s0 = min(c1, c0 + lane * per), s1 = min(c1, s0 + per);
    double seg = 0.0;
#pragma unroll 4
    for (int v = s0; v < s1; ++v) seg += w(v);
    double sincl = seg;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double y = __shfl_up(sincl, o, 64);
        if (lane >= o) sincl += y;
    }
    const unsigned long long hit = __ballot(base + sincl > target);
    int tok = -1;
    if (hit) {
        const int hl = __ffsll((long long)hit) - 1;
        double before = base + __shfl(sincl - seg, hl, 64);  // running sum in front of that segment
        const int h0 = min(c1, c0 + hl * per), h1 = min(c1, h0 + per);
        for (int v0 = h0; v0 < h1 && tok < 0; v0 += 64) {
            const int v = v0 + lane;
            const double x = v < h1 ? w(v) : 0.0;
            double ix = x;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const double y = __shfl_up(ix, o, 64);
                if (lane >= o) ix += y;
            }
            const unsigned long long h2 = __ballot(before + ix > target);
            if (h2) tok = v0 + __ffsll((long long)h2) - 1;
            before += __shfl(ix, 63, 64);
        }
    }
    // the chunk sum crossed but, in this summation order, no prefix did: its last positive id
    return tok >= 0 ? tok : owner_last;
}

template <bool NUC>
__global__ __launch_bounds__(64) void sample_locate_kernel(SampleArgs a, SpreadBuf b, int self_commit, int32_t* prefix_len) {
    const int i = blockIdx.x;
    // the chunk records of both kinds of weights are requested before anything is known about the sequence
    const double* sums = b.sums + (size_t)i * b.chunks() * 2;
    const int32_t* last = b.last + (size_t)i * b.chunks() * 2;
    double xr[SPREAD_GROUPS64], xp[SPREAD_GROUPS64];
    int lr[SPREAD_GROUPS64], lq[SPREAD_GROUPS64];
#pragma unroll
    for (int g = 0; g < SPREAD_GROUPS64; ++g) {
        const int c = g * 64 + (int)threadIdx.x;
        const bool in = c < b.chunks();
        const int cc = in ? c : 0;
        xr[g] = sums[cc * 2];
        xp[g] = sums[cc * 2 + 1];
        lr[g] = last[cc * 2];
        lq[g] = last[cc * 2 + 1];
        if (!in) {
            xr[g] = 0.0;
            xp[g] = 0.0;
            lr[g] = -1;
            lq[g] = -1;
        }
    }
    const int acc_len = a.accept_len[i];
    const double* rs = b.row_stats + 2 * (a.judge_index(i, acc_len) + 1);
    const TokenWeights<NUC> w(a, i, acc_len, rs[0], rs[1]);
    const double u = (double)a.u[i * (a.k + 1) + a.k];
    int tok = -1;
    if (w.qrow) {
        auto rw = [&](int v) { return w.r(w.p(v), v); };
        tok = wave_inverse_cdf(rw, a.V, u, xr, lr, b.chunks(), b.chunk);
    }
    if (tok < 0) {  // bonus token, or the residual vanished (p == q): draw from p
        auto pw = [&](int v) { return w.p(v); };
        tok = wave_inverse_cdf(pw, a.V, u, xp, lq, b.chunks(), b.chunk);
    }
    if (threadIdx.x == 0) {
        a.next_token[i] = tok;
        if (self_commit) {
            if (status_now(a.status) != 0) {
                write_failed_commit(a.commit, prefix_len, a.P);
            } else {
                a.commit[0] = 0;
                a.commit[1] = acc_len;
                a.commit[2] = tok;
                a.commit[3] = a.P + a.R + acc_len;
                if (prefix_len) *prefix_len = a.P + a.R + acc_len;
            }
        }
    }
}

// The sequential first-token rule of Alg. 2 over s candidate sequences: p_run (already filled with the
// judging distribution) is tested against each first token in index order and replaced by its normalised
// residual after every rejection.  Returns the accepted sequence or -1 (same value in every thread).
// Candidate i has token first_tok[i * tok_stride], draft distribution first_q + i * q_stride, uniform
// first_u[i * u_stride].
__device__ int sequential_first_tokens(double* p_run, int V, int s, const int32_t* first_tok, int tok_stride,
                                       const float* first_q, size_t q_stride, const float* first_u, int u_stride,
                                       double* sm_d) {
    const int tid = threadIdx.x;
    for (int i = 0; i < s; ++i) {
        int t = first_tok[i * tok_stride];
        t = t < 0 ? 0 : (t >= V ? V - 1 : t);
        const float* qrow = first_q + (size_t)i * q_stride;
        const double lhs = (double)first_u[i * u_stride] * (double)qrow[t];
        if (lhs < p_run[t]) return i;  // same value in every thread
        double sum = 0.0;
        for (int v = tid; v < V; v += SAMPLE_THREADS) sum += fmax(p_run[v] - (double)qrow[v], 0.0);
        const double Rm = block_sum_d(sum, sm_d);
        if (Rm > 0.0)
            for (int v = tid; v < V; v += SAMPLE_THREADS) p_run[v] = fmax(p_run[v] - (double)qrow[v], 0.0) / Rm;
        __syncthreads();
    }
    return -1;
}

template <bool NUC>
__global__ __launch_bounds__(SAMPLE_THREADS) void sample_paper_kernel(SampleArgs a) {
    __shared__ double sm_d[16];
    __shared__ int sm_i[4 + 16];
    __shared__ double sm_st[DUO_MAX_ROWS + 1][2];
    const SeqStats st{sm_st};
    const int tid = threadIdx.x;
    load_seq_stats(a, 0, 0, 0, st);  // the distribution that judges every first token
    fill_running_distribution<NUC>(a, st, 0, 0);
    const int sel = sequential_first_tokens(a.p_run, a.V, a.n, a.tokens, a.k, a.q, (size_t)a.k * a.V, a.u, a.k + 1, sm_d);
    int acc_len = 0, tok;
    if (sel < 0) {
        const double* pr = a.p_run;
        auto pw = [=](int v) { return pr[v]; };
        tok = block_inverse_cdf(pw, a.V, (double)a.u[(a.n - 1) * (a.k + 1) + a.k], sm_d, sm_i);
    } else {
        load_seq_stats(a, sel, 1, a.k, st);  // the rows of the selected sequence
        accept_flags<NUC>(a, st, sel, 1);
        acc_len = leading_accepts(a, sel, 1);
        tok = finish_token<NUC>(a, st, sel, acc_len, sm_d, sm_i);
    }
    for (int i = tid; i < a.n; i += SAMPLE_THREADS) {
        a.accept_len[i] = sel < 0 ? 0 : (i < sel ? 0 : (i == sel ? acc_len : -1));
        a.next_token[i] = i == sel ? tok : -1;
    }
    if (tid == 0) {
        a.commit[0] = sel;
        a.commit[1] = acc_len;
        a.commit[2] = tok;
        a.commit[3] = a.P + a.R + acc_len;
    }
}

// Alg. 2 as listed (one round of the pipelined loop): the k = l rows of the single sequence are the
// unverified suffix; after it, only the first tokens of s new sequences are judged.  One workgroup.
struct DeferredArgs {
    const int32_t* first_tokens;  // [s]
    const float* first_probs;     // [s][V]
    const float* uniforms_first;  // [s]
    int s;
    int32_t* prefix_len;  // device prefix length to advance, may be NULL (sampling only)
};

template <bool NUC>
__global__ __launch_bounds__(SAMPLE_THREADS) void sample_deferred_kernel(SampleArgs a, DeferredArgs d) {
    __shared__ double sm_d[16];
    __shared__ int sm_i[4 + 16];
    __shared__ double sm_st[DUO_MAX_ROWS + 1][2];
    const SeqStats st{sm_st};
    const int tid = threadIdx.x;
    if (tid < d.s && a.status) {
        const int t = d.first_tokens[tid];
        if (t < 0 || t >= a.V) atomicOr(a.status, 1);
    }
    load_seq_stats(a, 0, 0, a.k, st);
    accept_flags<NUC>(a, st, 0, 0);
    const int acc_len = leading_accepts(a, 0, 0);
    int sel = -1, tok = -1;
    if (acc_len < a.k) {
        tok = finish_token<NUC>(a, st, 0, acc_len, sm_d, sm_i);  // residual draw at the first rejection
    } else {
        fill_running_distribution<NUC>(a, st, 0, a.k);  // the distribution after the last scored token
        sel = sequential_first_tokens(a.p_run, a.V, d.s, d.first_tokens, 1, d.first_probs, (size_t)a.V, d.uniforms_first, 1,
                                      sm_d);
        if (sel < 0) {
            const double* pr = a.p_run;
            auto pw = [=](int v) { return pr[v]; };
            tok = block_inverse_cdf(pw, a.V, (double)a.u[a.k], sm_d, sm_i);
        }
    }
    if (tid == 0) {  // the flags of this kernel's own token check were set before the barriers above
        a.accept_len[0] = acc_len;
        a.next_token[0] = tok;
        if (status_now(a.status) != 0) {
            write_failed_commit(a.commit, d.prefix_len, a.P);
        } else {
            a.commit[0] = sel;
            a.commit[1] = acc_len;
            a.commit[2] = tok;
            a.commit[3] = a.P + a.R + acc_len;
            if (d.prefix_len) *d.prefix_len = a.P + a.R + acc_len;
        }
    }
}

struct CommitArgs {
    u16* kc;  // [L][Hkv] planes of max_seq * D elements, tiled layouts (k_cache_offset, v_cache_offset)
    u16* vc;
    int Hkv, D, max_seq;
    int P, R, n, k, mode;
    const int32_t* accept_len;
    const int32_t* next_token;
    int32_t* commit;
    int32_t* prefix_len;  // may be NULL (sampling only)
    int32_t* status;
};

// grid (Hkv, L) for the copy; (1, 1) when there is no cache.  In longest mode every workgroup
// recomputes the (cheap) selection; workgroup (0, 0) publishes it.  A pass whose status word is not clean moves
// nothing and leaves the prefix length alone.
__global__ __launch_bounds__(256) void commit_kernel(CommitArgs a) {
    if (status_now(a.status) != 0) {  // same value in every workgroup: all flags were set by earlier kernels
        if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) write_failed_commit(a.commit, a.prefix_len, a.P);
        return;
    }
    int sel, len, tok;
    if (a.mode == 0) {
        sel = 0;
        len = a.accept_len[0];
        for (int i = 1; i < a.n; ++i)
            if (a.accept_len[i] > len) {
                len = a.accept_len[i];
                sel = i;
            }
        tok = a.next_token[sel];
    } else {
        sel = a.commit[0];
        len = a.commit[1];
        tok = a.commit[2];
    }
    const int newP = a.P + a.R + len;
    if (a.kc && sel > 0 && len > 0) {
        const int hk = blockIdx.x, l = blockIdx.y;
        const int src = a.P + a.R + sel * a.k, dst = a.P + a.R;
        u16* kp = a.kc + ((size_t)l * a.Hkv + hk) * a.max_seq * a.D;
        u16* vp = a.vc + ((size_t)l * a.Hkv + hk) * a.max_seq * a.D;
        // source rows [src, src + len) and destination rows [dst, dst + len) never overlap: src - dst = sel * k >= len
        for (int e = threadIdx.x; e < len * a.D; e += 256) {
            const int j = e / a.D, d = e - j * a.D;
            kp[k_cache_offset(a.D, dst + j, d)] = kp[k_cache_offset(a.D, src + j, d)];
            vp[v_cache_offset(a.D, dst + j, d)] = vp[v_cache_offset(a.D, src + j, d)];
        }
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        if (a.mode == 0) {
            a.commit[0] = sel;
            a.commit[1] = len;
            a.commit[2] = tok;
            a.commit[3] = newP;
        }
        if (a.prefix_len) *a.prefix_len = newP;
    }
}

// Prefill bookkeeping: all m rows join the prefix, the last row's logits become the root logits.  Nothing is
// changed when the pass's status word is not clean.
__global__ void prefill_finish_kernel(const float* __restrict__ last_logits, float* __restrict__ root_logits, int V,
                                      int32_t* prefix_len, int newP, int32_t* status) {
    if (status_now(status) != 0) return;
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v < V) root_logits[v] = last_logits[v];
    if (v == 0) *prefix_len = newP;
}
