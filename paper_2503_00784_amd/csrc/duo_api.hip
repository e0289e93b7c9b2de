// C ABI of the verify step: host-side validation, workspace carving and the launch sequence.
// Everything that computes lives in the kernels of duo_gemm.h / duo_attn.h / duo_rowops.h /
// duo_sample.h; this file only enqueues them on the caller's stream.
#include "../../include/duo_verify.h"

#include <math.h>
#include <algorithm>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "duo_attn.h"
#include "duo_common.h"
#include "duo_gemm.h"
#include "duo_gemm_block.h"
#include "duo_pack.h"
#include "duo_rowops.h"
#include "duo_sample.h"

// ---- scratch of the entry point that allocates nothing (duo_spec_sample_noalloc): what duo_spec_sample takes from its
// workspace argument, sized for DUO_NOALLOC_MAX_VOCAB and without the nucleus search rows.  The array lives in every
// device's copy of this code object; host code never passes its name to a kernel, only the per-device address that
// hipGetSymbolAddress returned.
constexpr size_t NOALLOC_STATS_BYTES = (size_t)2 * DUO_MAX_ROWS * STATS_SPLIT * 2 * sizeof(double);
constexpr size_t NOALLOC_PRUN_BYTES = (size_t)DUO_NOALLOC_MAX_VOCAB * sizeof(double);
constexpr size_t NOALLOC_ACC_BYTES = 512;  // DUO_MAX_ROWS accept flags
static_assert(NOALLOC_STATS_BYTES % 256 == 0 && NOALLOC_PRUN_BYTES % 256 == 0 && DUO_MAX_ROWS * sizeof(int32_t) <= NOALLOC_ACC_BYTES,
              "the three parts keep the array's alignment");
static_assert(((size_t)(DUO_MAX_ROWS + 1) * STATS_SPLIT + ROOT_STATS_PARTS) * 2 * sizeof(double) <= NOALLOC_STATS_BYTES,
              "row and root statistics fit their part");
constexpr size_t NOALLOC_SCRATCH_BYTES = NOALLOC_STATS_BYTES + NOALLOC_PRUN_BYTES + NOALLOC_ACC_BYTES;
static_assert(NOALLOC_SCRATCH_BYTES == DUO_NOALLOC_SCRATCH_BYTES, "the header states the array's size");
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

namespace {

thread_local char g_hip_err[256] = "";

int hip_ok(hipError_t e, const char* what) {
    if (e == hipSuccess) return DUO_OK;
    snprintf(g_hip_err, sizeof g_hip_err, "%s: %s", what, hipGetErrorString(e));
    return DUO_ERR_HIP;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

constexpr int MAX_CHUNKS = 64;
constexpr int MAX_CHUNKS_MANY_ROWS = 8;  // key chunks of the attention kernels in passes of more than DUO_MAX_ROWS rows

// K splits of a residual projection (N = d_model columns) in the many-row pass: enough workgroups of 128 x 128 for
// the chip, at most eight partial results.
int block_splits(int M, int N) {
    const int mh = pair_rows_for(M) / 16;
    const int wgs = ((N / 16 + 7) / 8) * ((mh + 7) / 8);
    const int S = 256 / wgs;
    return S < 1 ? 1 : (S > WIDE_MAX_SPLIT ? WIDE_MAX_SPLIT : S);
}

// GEMM operand buffers (h, attn, act) hold activations as bf16 pairs: row m = hi, row pair_rows + m = lo,
// padded to whole 16-row MFMA tiles; rows that carry no activation are never stored from.
constexpr int QKV_SPLITS = 4;  // most K splits of the Q/K/V projection at 49..80 rows (QkvFinishArgs::MAX_SPLITS)

struct Workspace {
    float* x;        // fp32 residual stream [M][d]
    u16* h;          // normalised activations, operand layout [A_rows][d]
    u16* q;          // rotated queries: hi plane [Mp][Hq*D], lo plane [Mp][Hq*D]
    u16* attn;       // attention output, operand layout [A_rows][Hq*D]
    u16* act;        // SwiGLU output, operand layout [A_rows][F]
    float* part;     // attention chunk partials
    float* rope_c;   // [Mp][D/2]
    float* rope_s;
    float* logits;   // fp32 [Mp][V]
    double* stats_rows;  // sampler: partial softmax statistics [DUO_MAX_ROWS + 1][stats_parts][2]
    double* stats_root;  // [STATS_SPLIT][2]
    int stats_parts;
    double* p_run;
    double* nuc;     // nucleus records [DUO_MAX_ROWS + 1][4]
    double* p_rows;  // nucleus search scratch [DUO_MAX_ROWS + 1][vocab]
    int32_t* acc;
    float* ssq;      // [Mp][d/16] partial sums of squares of the residual stream (for the next RMSNorm)
    float* ssq_full; // [Mp][RowScale::FULL_PARTS] sums of squares over column ranges (written by the few-workgroups-per-row producers)
    float* split;    // [splits][Mp][d] partial results of the K-split residual projections; [2][M][Q/K/V columns] of the K-split Q/K/V projection
    size_t split_floats;
    u16* h_last;     // many-row pass: the last row of h as an operand of its own (one tile per K step)
    size_t q_plane;  // elements between the two query planes
    size_t total;
};

// Partial statistics per judging row: the LM head's epilogue leaves one part per tile of 32 vocabulary entries, the
// statistics kernel of the sampling-only entry points STATS_SPLIT parts.
int lm_head_parts(int vocab) { return (vocab + 31) / 32; }
size_t stats_bytes(int parts) {
    return align_up((size_t)(DUO_MAX_ROWS + 1) * parts * 2 * sizeof(double), 256) + align_up((size_t)ROOT_STATS_PARTS * 2 * sizeof(double), 256);
}

size_t sample_ws_bytes(int vocab, int parts = STATS_SPLIT) {
    return stats_bytes(parts) + align_up((size_t)vocab * sizeof(double), 256) +
           align_up((size_t)DUO_MAX_ROWS * sizeof(int32_t), 256) + align_up((size_t)(DUO_MAX_ROWS + 1) * 4 * sizeof(double), 256) +
           align_up((size_t)(DUO_MAX_ROWS + 1) * vocab * sizeof(double), 256);
}

void carve_sampler(char* base, size_t& off, int vocab, Workspace& ws, int parts = STATS_SPLIT) {
    ws.stats_parts = parts;
    ws.stats_rows = reinterpret_cast<double*>(base + off);
    off += align_up((size_t)(DUO_MAX_ROWS + 1) * parts * 2 * sizeof(double), 256);
    ws.stats_root = reinterpret_cast<double*>(base + off);
    off += align_up((size_t)ROOT_STATS_PARTS * 2 * sizeof(double), 256);
    ws.p_run = reinterpret_cast<double*>(base + off);
    off += align_up((size_t)vocab * sizeof(double), 256);
    ws.acc = reinterpret_cast<int32_t*>(base + off);
    off += align_up((size_t)DUO_MAX_ROWS * sizeof(int32_t), 256);
    ws.nuc = reinterpret_cast<double*>(base + off);
    off += align_up((size_t)(DUO_MAX_ROWS + 1) * 4 * sizeof(double), 256);
    ws.p_rows = reinterpret_cast<double*>(base + off);
    off += align_up((size_t)(DUO_MAX_ROWS + 1) * vocab * sizeof(double), 256);
}

Workspace carve(const duo_model_config& c, int max_rows, void* base_v) {
    Workspace ws{};
    char* base = static_cast<char*>(base_v);
    const size_t Mp = align_up((size_t)max_rows, 16);
    const size_t Ar = (size_t)a_tiles_for(max_rows, true) * 16;
    const size_t d = c.d_model, qd = (size_t)c.n_q_heads * c.head_dim, F = c.d_ff, V = c.vocab;
    const size_t group = c.n_q_heads / c.n_kv_heads;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = base + off;
        off += align_up(bytes, 256);
        return p;
    };
    ws.x = reinterpret_cast<float*>(take(Mp * d * 4));
    ws.h = reinterpret_cast<u16*>(take(Ar * d * 2));
    ws.q_plane = Mp * qd;
    ws.q = reinterpret_cast<u16*>(take(2 * Mp * qd * 2));
    ws.attn = reinterpret_cast<u16*>(take(Ar * qd * 2));
    ws.act = reinterpret_cast<u16*>(take(Ar * F * 2));
    const bool many = max_rows > DUO_MAX_ROWS;  // prefill pass: few key chunks, logits of the last row only
    ws.part = reinterpret_cast<float*>(
        take((size_t)c.n_kv_heads * (Mp * group) * (many ? MAX_CHUNKS_MANY_ROWS : MAX_CHUNKS) * (c.head_dim + 4) * 4));
    ws.rope_c = reinterpret_cast<float*>(take(Mp * (c.head_dim / 2) * 4));
    ws.rope_s = reinterpret_cast<float*>(take(Mp * (c.head_dim / 2) * 4));
    ws.logits = reinterpret_cast<float*>(take((many ? 16 : Mp) * V * 4));
    ws.ssq = reinterpret_cast<float*>(take(Mp * (d / 16) * 4));
    ws.ssq_full = reinterpret_cast<float*>(take(Mp * RowScale::FULL_PARTS * 4));
    ws.split_floats = (size_t)(many ? block_splits(max_rows, c.d_model) : WIDE_MAX_SPLIT) * Mp * d;
    if (!many) ws.split_floats = std::max(ws.split_floats, (size_t)QKV_SPLITS * Mp * (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim);
    ws.split = reinterpret_cast<float*>(take(ws.split_floats * 4));
    ws.h_last = reinterpret_cast<u16*>(take(16 * d * 2));
    carve_sampler(base, off, c.vocab, ws, lm_head_parts(c.vocab));
    ws.total = off;
    return ws;
}

int check_config(const duo_model_config* c) {
    if (!c) return DUO_ERR_NULL;
    if (c->n_layers < 1 || c->d_model < 32 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ff < 32 || c->vocab < 2 ||
        c->max_seq < 32)
        return DUO_ERR_SHAPE;
    if (c->head_dim != 64 && c->head_dim != 128) return DUO_ERR_SHAPE;
    if (c->d_model % 64 || c->d_model > 8192 || c->d_ff % 32 || c->max_seq % 32) return DUO_ERR_SHAPE;
    if (c->n_q_heads % c->n_kv_heads || c->n_q_heads > 512) return DUO_ERR_SHAPE;
    if (!(c->rope_theta > 0.f) || !(c->rms_eps >= 0.f)) return DUO_ERR_SHAPE;
    return DUO_OK;
}

int check_weights(const duo_model_config* c, const duo_weights* w) {
    if (!w || !w->embed || !w->wqkv || !w->wo || !w->w_gate_up || !w->w_down || !w->g_attn || !w->g_ffn || !w->g_final ||
        !w->lm_head)
        return DUO_ERR_NULL;
    if (!aligned16(w->embed) || !aligned16(w->lm_head) || !aligned16(w->g_final)) return DUO_ERR_ALIGN;
    const uint16_t* const* tabs[6] = {w->wqkv, w->wo, w->w_gate_up, w->w_down, w->g_attn, w->g_ffn};
    for (auto tab : tabs)
        for (int l = 0; l < c->n_layers; ++l) {
            if (!tab[l]) return DUO_ERR_NULL;
            if (!aligned16(tab[l])) return DUO_ERR_ALIGN;
        }
    return DUO_OK;
}

// ---- optional per-kernel timing (see duo_profile_enable in the header)
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> ev;  // pairs: start, stop
    std::vector<int> cls;        // class of pair i
    size_t used = 0;             // pairs in use
    size_t dropped = 0;          // launches since the last read that found the pool empty
    char names[DUO_PROF_CLASSES][128] = {};  // per class: the kernel last launched under it, as its launch helper spelled it
};
Profiler g_prof;
constexpr size_t PROF_POOL = 8192;  // pairs

// Called right before a launch of class `cls`: arms DUO_LAUNCH with the next event pair.
inline void prof(int cls, hipStream_t) {
    if (!g_prof.on || cls < 0) return;
    if (g_prof.used >= g_prof.cls.size()) {
        ++g_prof.dropped;
        return;
    }
    g_launch_events.start = g_prof.ev[2 * g_prof.used];
    g_launch_events.stop = g_prof.ev[2 * g_prof.used + 1];
    g_launch_events.name = cls < DUO_PROF_CLASSES ? g_prof.names[cls] : nullptr;
    g_prof.cls[g_prof.used] = cls;
    ++g_prof.used;
}

template <int D>
void launch_attention(int mtw, int nwv, dim3 grid, const AttnArgs& a, hipStream_t s) {
    if (nwv == 8) {
        if (mtw == 1) DUO_LAUNCH((attn_partial_kernel<D, 1, 8>), grid, dim3(512), s, a);
        else if (D == 64) DUO_LAUNCH((attn_partial_kernel<64, 2, 8>), grid, dim3(512), s, a);
    } else {
        if (mtw == 1) DUO_LAUNCH((attn_partial_kernel<D, 1, 4>), grid, dim3(256), s, a);
        else DUO_LAUNCH((attn_partial_kernel<D, 2, 4>), grid, dim3(256), s, a);
    }
}

// A projection whose epilogue finishes the rows (QKV, gate/up, LM head).  Up to eight rows every wave streams
// its own bands and reads the activations itself; beyond that the waves of a workgroup share the activation
// operand through LDS.
// `cls`: the kernel class of the per-kernel timer.
template <int NT, class Epi>
void launch_projection(int cls, int M, const u16* X, const u16* W, int K, int tiles, const RowScale& rsc, const Epi& epi,
                       hipStream_t s) {
    if (M > DUO_MAX_ROWS) {  // prefill pass: both operands staged in LDS; wider blocks once they still fill the chip
        launch_block_rows<NT>(X, W, K, tiles * NT, M, rsc, epi, s, [&]() { prof(cls, s); });
        return;
    }
    prof(cls, s);
    if (M <= 8) {
        if (!launch_wide_half<NT>(X, W, K, tiles, rsc, epi, s)) launch_gemm_rows<NT>(M, true, X, W, K, tiles, rsc, epi, s);
        return;
    }
    const int quads = pair_rows_for(M) / 4;
    switch ((M + 15) / 16) {
        case 1: launch_wide<1, NT>(X, W, K, tiles, quads, rsc, epi, s); break;
        case 2: launch_wide<2, NT>(X, W, K, tiles, quads, rsc, epi, s); break;
        case 3: launch_wide<3, NT>(X, W, K, tiles, quads, rsc, epi, s); break;
        case 4: launch_wide<4, NT>(X, W, K, tiles, quads, rsc, epi, s); break;
        default: launch_wide<5, NT>(X, W, K, tiles, quads, rsc, epi, s); break;
    }
}

// x += act W^T (O and down projections, N = d_model columns) followed by the preparation of the next RMSNorm.
// Few rows: one kernel (EpiResidual).  Many rows: K split over workgroups, partial results, and a small
// second kernel that adds them in split order and does EpiResidual's work.
static_assert(WIDE_MAX_SPLIT <= 8, "residual_reduce_kernel holds at most eight splits in registers");

// Whether the residual projection over K input channels runs as K-split partial products + reduce kernel: beyond 16
// rows.  (At 32 rows x 4096 input channels the split form alone is no faster, 10.3 + 4.2 against 14.0 us, but the reduce
// kernel leaves whole-row sums of squares, which the next projection turns into its factors 2.5 us sooner than the 256
// partial sums per row of the one-kernel form: 3.62 -> 3.53 ms per step at 32 rows of the 7B shape.)
bool residual_is_split(int M, int /*K*/, int N) {
    if (M > DUO_MAX_ROWS) return block_splits(M, N) > 1;
    return M > 16;
}

void launch_residual_projection(int M, const u16* X, const u16* W, int K, const EpiResidual& er, float* split,
                                float* ssq_full, int cls, hipStream_t s) {
    const RowScale none{nullptr, 0, 0.f, 0.f, nullptr};
    const int MH = (M + 15) / 16, d = er.N;
    if (!residual_is_split(M, K, d)) {
        prof(cls, s);
        if (M > DUO_MAX_ROWS) launch_block<4, 4, 1>(X, W, K, d / 16, M, 1, none, er, s);
        else launch_gemm_rows<1>(M, true, X, W, K, d / 16, none, er, s);
        return;
    }
    int S = 1;
    prof(cls, s);
    if (M > DUO_MAX_ROWS) {
        EpiStoreF32 e{d, M, 1, split, d, (size_t)M * d};
        S = launch_block<4, 4, 1>(X, W, K, d / 16, M, block_splits(M, d), none, e, s);
    } else switch (MH) {
        case 2: S = launch_wide_split<2>(X, W, K, d, M, split, none, s); break;
        case 3: S = launch_wide_split<3>(X, W, K, d, M, split, none, s); break;
        case 4: S = launch_wide_split<4>(X, W, K, d, M, split, none, s); break;
        default: S = launch_wide_split<5>(X, W, K, d, M, split, none, s); break;
    }
    prof(DUO_PROF_RESID_REDUCE, s);
    launch_residual_reduce(M, split, S, (size_t)M * d, er.X, er.gain, er.h, d, er.pair_rows, er.h_tiles, er.ssq_part, ssq_full, s);
}

template <int D>
void launch_attention_shared(int mtw, int nwv, int ksplit, dim3 grid, const AttnArgs& a, hipStream_t s) {
    if (mtw == 2) DUO_LAUNCH((attn_shared_kernel<D, 2, 7>), grid, dim3(512), s, a);  // 8 waves: 256 registers each
    else if (ksplit == 2 && nwv == 8) DUO_LAUNCH((attn_shared_kernel<D, 1, 8, 2>), grid, dim3(576), s, a);
    else if (ksplit == 2) DUO_LAUNCH((attn_shared_kernel<D, 1, 4, 2>), grid, dim3(320), s, a);
    else DUO_LAUNCH((attn_shared_kernel<D, 1, 8>), grid, dim3(576), s, a);
}

// The target pass over the rows of `plan`: fills the cache slots P .. P+M-1 and writes fp32
// logits [M][V] (row stride V) to `logits`.
// `temperature` >= 0: the pass is followed by sampling at that temperature, so the LM head also leaves the softmax
// statistics of its rows (ws.stats_rows) and, without a root row, the first kernel those of the cached root logits
// (ws.stats_root); < 0: logits only.
void enqueue_forward(const duo_model_config& c, const duo_weights& w, const duo_kv_cache& cache,
                     const int32_t* tokens, int root_token, const RowPlan& plan, const Workspace& ws,
                     float* logits, int32_t* status, hipStream_t s, double temperature = -1.0) {
    const int M = plan.M, Mp = (M + 15) / 16 * 16, PR = pair_rows_for(M), AT = a_tiles_for(M, true);
    const int d = c.d_model, D = c.head_dim, half = D / 2, Hq = c.n_q_heads, Hkv = c.n_kv_heads;
    const int qd = Hq * D, F = c.d_ff, V = c.vocab, group = Hq / Hkv;

    const int NP = d / 16;  // partial sums of squares per row (one per 16-column tile of the residual stream)
    // RMSNorm factors from the producer's partial sums, or from its complete row sums where it wrote them
    // (embedding gather, K-split reduce) and the consumer is the LDS-shared kernel, which reads them directly.
    const RowScale norm_part{ws.ssq, NP, 1.0f / (float)d, c.rms_eps, nullptr};
    const RowScale norm_full{ws.ssq, NP, 1.0f / (float)d, c.rms_eps, ws.ssq_full};
    const bool o_split = residual_is_split(M, qd, d), down_split = residual_is_split(M, F, d);
    const bool many = M > DUO_MAX_ROWS;  // prefill pass: logits of the last row only (to logits[0 .. V))
    const int max_chunks = many ? MAX_CHUNKS_MANY_ROWS : MAX_CHUNKS;
    const bool stats = temperature >= 0.0;
    const bool root_stats = stats && plan.R == 0;
    prof(DUO_PROF_SETUP, s);
    DUO_LAUNCH(rope_table_kernel, dim3(M + (root_stats ? ROOT_STATS_PARTS : 0)), dim3(256), s, plan, D, (double)c.rope_theta, ws.rope_c,
               ws.rope_s, status, RootStatsArgs{root_stats ? cache.root_logits : nullptr, V, temperature, ws.stats_root});
    prof(DUO_PROF_SETUP, s);
    DUO_LAUNCH(embed_kernel, dim3(M), dim3(256), s, w.embed, tokens, root_token, plan, V, cache.prefix_len,
                       status, ws.x, w.g_attn[0], ws.h, d, PR, AT, ws.ssq, ws.ssq_full);

    // Attention launch shape.  Short contexts: one workgroup of 8 waves per (kv head, row group) does
    // the whole head and writes the output itself.  Long contexts: the keys are cut into chunks for
    // more workgroups, and a second small kernel merges the chunk partials.
    const int Ktot = plan.P + M;
    const int NB = (Ktot + 31) / 32;
    const int MQ = M * group, MqT = (MQ + 15) / 16;
    const int mtw = MqT >= 2 ? 2 : 1;
    const int MG = (MqT + mtw - 1) / mtw;
    const int mq_pad = Mp * group;
    // Two or more query tiles per kv head: the kernel that stages K/V blocks in LDS for all query tiles
    // (two tiles on a short context stay with the per-wave kernel, which then needs no chunk merge).
    const bool shared_kv = MqT > 2 || (MqT == 2 && NB > 32);
    int sh_mtw = 1, sh_nwv = 4, sh_zg = 1, sh_ksplit = 1;
    int nwv, bpw, nchunks;
    if (shared_kv) {
        // one query tile per wave, about 256 workgroups (one per compute unit): measured best for 4 tiles x 32 heads and 16 tiles x 8 heads
        // Up to four tiles: two teams of waves share the blocks (two waves per SIMD: 20.7 against 23.2 us at 4 tiles,
        // 11.8 against 14.4 us at 2 tiles, measured on 32 heads x 4160 / 2080 keys).
        sh_mtw = MqT > 16 ? 2 : 1;
        sh_ksplit = (MqT <= 4 || (MqT > 8 && MqT <= 16)) ? 2 : 1;  // 9..16 tiles (64 rows x a GQA group of 4): 27.3 against 28.2 us at 8192 keys
        sh_nwv = MqT > 16 ? 7 : (MqT > 2 ? 8 : 4);
        sh_zg = (MqT + (sh_nwv / sh_ksplit) * sh_mtw - 1) / ((sh_nwv / sh_ksplit) * sh_mtw);
        int target = (256 + Hkv * sh_zg - 1) / (Hkv * sh_zg);
        target = target < 1 ? 1 : (target > max_chunks ? max_chunks : target);
        if (many) {
            // many row groups: the chunk count that leaves the fewest compute units idle in the last round of
            // workgroups (160 (head, row group) pairs: 3 chunks = 480 workgroups, not 2 = 320), few chunks preferred
            float best = -1.f;
            for (int t = 1; t <= max_chunks; ++t) {
                const int wgs = Hkv * sh_zg * t;
                const float eff = (float)wgs / (float)((wgs + 255) / 256 * 256) - 0.04f * (float)t;
                if (eff > best) {
                    best = eff;
                    target = t;
                }
            }
        }
        bpw = (NB + target - 1) / target;  // blocks per chunk
        bpw = bpw < 2 ? 2 : bpw;
        nchunks = (NB + bpw - 1) / bpw;
        nwv = sh_nwv;
    } else if (NB <= 32) {
        nwv = (mtw == 2 && D == 128) ? 4 : 8;  // register budget of the two-tile, 128-channel variant
        bpw = (NB + nwv - 1) / nwv;
        nchunks = 1;
    } else {
        // about 224 workgroups, at least two blocks per wave (measured on 32 heads x 2080 keys: 192 workgroups
        // of 3 blocks per wave take 14 us, 544 of one block 24 us)
        nwv = 4;
        int target = (224 + Hkv * MG - 1) / (Hkv * MG);
        target = target < 1 ? 1 : (target > max_chunks ? max_chunks : target);
        bpw = (NB + 4 * target - 1) / (4 * target);
        bpw = bpw < 2 ? 2 : bpw;
        nchunks = (NB + 4 * bpw - 1) / (4 * bpw);
    }

    // The bands of the Q/K/V matrix are independent of each other, so a wave may take one or two.  One band per wave
    // where that makes a single, nearly full round of workgroups (measured at 768 bands of 4096 input channels:
    // 18.5 against 21.1 us for up to eight rows, 18.8 / 21.8 / 28.7 / 32.4 against 22.0 / 24.8 / 32.1 / 35.2 us for
    // 16 / 32 / 64 / 80 rows; at 384 bands the same or slightly better beyond eight rows).
    const int qkv_bands = (Hq + 2 * Hkv) * (D / 16);
    const int qkv_nt = M > DUO_MAX_ROWS ? 2 : (M <= 8 ? ((qkv_bands > 512 && qkv_bands <= 768) ? 1 : 2) : (qkv_bands <= 768 ? 1 : 2));
    // the Q/K/V projection as K-split product + finish kernel (see the loop): 49..80 rows, one band per wave, partial results fit
    const bool qkv_split = M > 48 && M <= DUO_MAX_ROWS && qkv_nt == 1 && (size_t)QKV_SPLITS * M * qkv_bands * 16 <= ws.split_floats;
    for (int l = 0; l < c.n_layers; ++l) {
        u16* kc = cache.k + (size_t)l * Hkv * c.max_seq * D;
        u16* vc = cache.v + (size_t)l * Hkv * c.max_seq * D;
        EpiQKV eq{Hq, Hkv, D, half, D / 16, qkv_nt, ws.q, qd, ws.q_plane, kc, vc, c.max_seq, ws.rope_c, ws.rope_s, plan,
                  cache.prefix_len, 1};
        const RowScale& qkv_norm = (l == 0 || down_split) ? norm_full : norm_part;
        if (qkv_split) {
            // 49..80 rows: K split two or four ways over workgroups of as many times the bands, each staging its part of the
            // operand (22.1 against 27.1 us for the product at 64 rows x 768 bands), partial results to the workspace, and a
            // small second kernel that adds them and does the rotary embedding and the cache scatter
            const int ncols = qkv_bands * 16;
            EpiStoreF32 ep{ncols, M, 1, ws.split, ncols, (size_t)M * ncols};
            const int quads = pair_rows_for(M) / 4;
            int S = 1;
            prof(DUO_PROF_QKV, s);
            // (measured on one box: 768 bands, two splits of six-band workgroups 24.2 + 4.2 us against four splits of
            // twelve-band workgroups 26.6 + 5.5 us; 384 bands, four splits of six-band workgroups 15.2 + 4.6 us against
            // two splits of three-band workgroups 16.7 + 4.1 us)
            if (M <= 64) {
                if (qkv_bands > 512) launch_wide_cfg<4, 1, 6, 1>(ws.h, w.wqkv[l], d, qkv_bands, quads, 2, qkv_norm, ep, s, &S);
                else launch_wide_cfg<4, 1, 6, 1>(ws.h, w.wqkv[l], d, qkv_bands, quads, QKV_SPLITS, qkv_norm, ep, s, &S);
            } else {
                if (qkv_bands > 512) launch_wide_cfg<5, 1, 6, 1>(ws.h, w.wqkv[l], d, qkv_bands, quads, 2, qkv_norm, ep, s, &S);
                else launch_wide_cfg<5, 1, 6, 1>(ws.h, w.wqkv[l], d, qkv_bands, quads, QKV_SPLITS, qkv_norm, ep, s, &S);
            }
            QkvFinishArgs fa{ws.split, S, (size_t)M * ncols, ncols, Hq, Hkv, D, ws.q, qd, ws.q_plane, kc, vc, c.max_seq,
                             ws.rope_c, ws.rope_s, plan, cache.prefix_len};
            prof(DUO_PROF_QKV_FINISH, s);
            if (D == 128) DUO_LAUNCH(qkv_finish_kernel<128>, dim3(Hq + 2 * Hkv, (M + 7) / 8), dim3(256), s, fa);
            else DUO_LAUNCH(qkv_finish_kernel<64>, dim3(Hq + 2 * Hkv, (M + 7) / 8), dim3(256), s, fa);
        } else if (qkv_nt == 1) launch_projection<1>(DUO_PROF_QKV, M, ws.h, w.wqkv[l], d, qkv_bands, qkv_norm, eq, s);
        else launch_projection<2>(DUO_PROF_QKV, M, ws.h, w.wqkv[l], d, qkv_bands / 2, qkv_norm, eq, s);

        AttnArgs aa{ws.q, qd, ws.q_plane, kc, vc, c.max_seq, group, plan, Ktot, bpw, nchunks, mq_pad,
                    1.4426950408889634f / sqrtf((float)D), ws.part, ws.attn, AT, PR};
        prof(DUO_PROF_ATTN, s);
        if (shared_kv) {
            const dim3 grid(nchunks, Hkv, sh_zg);
            if (D == 128) launch_attention_shared<128>(sh_mtw, sh_nwv, sh_ksplit, grid, aa, s);
            else launch_attention_shared<64>(sh_mtw, sh_nwv, sh_ksplit, grid, aa, s);
        } else if (NB <= 32 && MqT == 1) {  // short context, one query tile: the no-loop kernel
            if (D == 128) DUO_LAUNCH((attn_small_kernel<128, 4>), dim3(1, Hkv), dim3(512), s, aa);
            else DUO_LAUNCH((attn_small_kernel<64, 4>), dim3(1, Hkv), dim3(512), s, aa);
        } else if (D == 128) {
            launch_attention<128>(mtw, nwv, dim3(nchunks, Hkv, MG), aa, s);
        } else {
            launch_attention<64>(mtw, nwv, dim3(nchunks, Hkv, MG), aa, s);
        }
        if (nchunks > 1) {
            prof(DUO_PROF_ATTN_COMB, s);
            if (D == 128) DUO_LAUNCH((attn_combine_kernel<128>), dim3((MQ + 3) / 4, Hkv), dim3(256), s, aa);
            else DUO_LAUNCH((attn_combine_kernel<64>), dim3((MQ + 3) / 4, Hkv), dim3(256), s, aa);
        }

        // the residual projections leave x, the next norm's operand u = x * gain and its partial sums
        EpiResidual eo{d, M, ws.x, d, w.g_ffn[l], ws.h, PR, AT, ws.ssq};
        launch_residual_projection(M, ws.attn, w.wo[l], qd, eo, ws.split, ws.ssq_full, DUO_PROF_OPROJ, s);

        EpiSwiGLU eg{F, M, ws.act, AT, PR};
        launch_projection<2>(DUO_PROF_GATEUP, M, ws.h, w.w_gate_up[l], d, F / 16, o_split ? norm_full : norm_part, eg, s);

        const u16* gnext = l + 1 < c.n_layers ? w.g_attn[l + 1] : w.g_final;
        EpiResidual ed{d, M, ws.x, d, gnext, ws.h, PR, AT, ws.ssq};
        launch_residual_projection(M, ws.act, w.w_down[l], F, ed, ws.split, ws.ssq_full, DUO_PROF_DOWN, s);
    }
    if (many) {
        prof(DUO_PROF_LMHEAD, s);
        DUO_LAUNCH(last_row_operand_kernel, dim3(d / 32), dim3(64), s, ws.h, M - 1, PR, AT, ws.h_last);
        const RowScale last{ws.ssq + (size_t)(M - 1) * NP, NP, 1.0f / (float)d, c.rms_eps, down_split ? ws.ssq_full + (size_t)(M - 1) * RowScale::FULL_PARTS : nullptr};
        EpiStoreF32 el{V, 1, 2, logits, V};
        launch_projection<2>(DUO_PROF_LMHEAD, 1, ws.h_last, w.lm_head, d, (V + 31) / 32, last, el, s);
        return;
    }
    if (stats) {
        EpiLogitsStats el{V, M, 2, logits, V, ws.stats_rows, ws.stats_parts, temperature};
        launch_projection<2>(DUO_PROF_LMHEAD, M, ws.h, w.lm_head, d, (V + 31) / 32, down_split ? norm_full : norm_part, el, s);
    } else {
        EpiStoreF32 el{V, M, 2, logits, V};
        launch_projection<2>(DUO_PROF_LMHEAD, M, ws.h, w.lm_head, d, (V + 31) / 32, down_split ? norm_full : norm_part, el, s);
    }
}

// Nucleus sampling is on for 0 < top_p < 1 at a positive temperature (at temperature 0 the distribution is one-hot).
bool nucleus_on(const duo_call* call) { return call->top_p > 0.f && call->top_p < 1.f && call->temperature > 0.f; }

// After the statistics: the nucleus of every judging row (sa.nuc is where the other kernels will look for it).
void enqueue_nucleus(const SampleArgs& sa, float top_p, const Workspace& ws, hipStream_t s) {
    if (!sa.nuc) return;
    prof(DUO_PROF_SAMPLE, s);
    if (sa.V <= 32 * SAMPLE_THREADS)
        DUO_LAUNCH(sample_nucleus_kernel<32>, dim3(1 + sa.n * sa.k), dim3(SAMPLE_THREADS), s, sa, (double)top_p, ws.p_rows, ws.nuc);
    else
        DUO_LAUNCH(sample_nucleus_kernel<0>, dim3(1 + sa.n * sa.k), dim3(SAMPLE_THREADS), s, sa, (double)top_p, ws.p_rows, ws.nuc);
}

// have_stats: the forward pass that produced the logits left their softmax statistics (and the root row's) already
void enqueue_sampling(const SampleArgs& sa, float top_p, const Workspace& ws, int mode, u16* kc, u16* vc,
                      const duo_model_config* c, int32_t* prefix_len, hipStream_t s, bool have_stats = false) {
    if (!have_stats) {
        prof(DUO_PROF_SAMPLE, s);
        DUO_LAUNCH(sample_stats_kernel, dim3(sa.R + sa.n * sa.k + (sa.R ? 0 : 1), STATS_SPLIT), dim3(256), s, sa);
    }
    enqueue_nucleus(sa, top_p, ws, s);
    prof(DUO_PROF_SAMPLE, s);
    if (mode == DUO_SELECT_INDEPENDENT_LONGEST) {
        // one sequence: nothing to choose and nothing to move, the finish kernel writes the commit itself
        const bool self_commit = sa.n == 1;
        if (sa.V >= SPREAD_MIN_VOCAB) {
            // large vocabulary: row statistics, slice sums and the search as three small kernels over many compute units
            int G = sa.V / 4096;
            G = std::min(G, std::min(SPREAD_MAX_SLICES, SPREAD_MAX_GROUPS / sa.n));
            G = std::max(G, 1);
            const int chunk = ((sa.V + 16 * G - 1) / (16 * G) + 63) / 64 * 64;
            static_assert(2 * (DUO_MAX_ROWS + 2) <= 256 && 256 + SPREAD_MAX_GROUPS * 16 * 3 <= SPREAD_MIN_VOCAB, "the records fit p_run");
            SpreadBuf sb{sa.p_run, sa.p_run + 256, reinterpret_cast<int32_t*>(sa.p_run + 256 + (size_t)sa.n * 16 * G * 2), G, chunk};
            // (letting every slice merge the statistics of its sequence's rows itself saves this launch and costs more:
            // 2 x 11.6 against 3 x 6.9 us at 9 rows of 1000 parts)
            DUO_LAUNCH(sample_row_stats_kernel, dim3(sa.R + sa.n * sa.k + 1), dim3(256), s, sa, sb);
            prof(DUO_PROF_SAMPLE, s);
            if (sa.nuc) DUO_LAUNCH(sample_spread_kernel<true>, dim3(sa.n, G), dim3(SAMPLE_THREADS), s, sa, sb);
            else DUO_LAUNCH(sample_spread_kernel<false>, dim3(sa.n, G), dim3(SAMPLE_THREADS), s, sa, sb);
            prof(DUO_PROF_SAMPLE, s);
            if (sa.nuc) DUO_LAUNCH(sample_locate_kernel<true>, dim3(sa.n), dim3(64), s, sa, sb, self_commit ? 1 : 0, prefix_len);
            else DUO_LAUNCH(sample_locate_kernel<false>, dim3(sa.n), dim3(64), s, sa, sb, self_commit ? 1 : 0, prefix_len);
        } else if (sa.nuc) DUO_LAUNCH(sample_finish_kernel<true>, dim3(sa.n), dim3(SAMPLE_THREADS), s, sa, self_commit ? 1 : 0, prefix_len);
        else DUO_LAUNCH(sample_finish_kernel<false>, dim3(sa.n), dim3(SAMPLE_THREADS), s, sa, self_commit ? 1 : 0, prefix_len);
        if (self_commit) return;
    } else {
        if (sa.nuc) DUO_LAUNCH(sample_paper_kernel<true>, dim3(1), dim3(SAMPLE_THREADS), s, sa);
        else DUO_LAUNCH(sample_paper_kernel<false>, dim3(1), dim3(SAMPLE_THREADS), s, sa);
    }
    CommitArgs ca{kc, vc, c ? c->n_kv_heads : 1, c ? c->head_dim : 0, c ? c->max_seq : 0, sa.P, sa.R, sa.n, sa.k, mode,
                  sa.accept_len, sa.next_token, sa.commit, prefix_len, sa.status};
    const dim3 grid = kc ? dim3(c->n_kv_heads, c->n_layers) : dim3(1, 1);
    prof(DUO_PROF_COMMIT, s);
    DUO_LAUNCH(commit_kernel, grid, dim3(256), s, ca);
}

// min_k: 1 for the fused step; 0 for the deferred form, whose unverified suffix may be empty
int check_call(const duo_call* call, int vocab, int min_k = 1) {
    if (!call) return DUO_ERR_NULL;
    if (call->n < 1 || call->k < min_k) return DUO_ERR_SHAPE;
    const int R = call->root_token >= 0 ? 1 : 0;
    if ((long long)call->n * call->k + R > DUO_MAX_ROWS) return DUO_ERR_SHAPE;
    if (!(call->temperature >= 0.f)) return DUO_ERR_ARG;  // 0 is the greedy limit; NaN fails the comparison
    if (call->top_p != call->top_p) return DUO_ERR_ARG;    // NaN
    if (call->select_mode != DUO_SELECT_INDEPENDENT_LONGEST && call->select_mode != DUO_SELECT_PAPER_SEQUENTIAL)
        return DUO_ERR_ARG;
    if (call->root_token >= vocab) return DUO_ERR_TOKEN_RANGE;
    if (call->host_prefix_len < 0) return DUO_ERR_ARG;
    return DUO_OK;
}

int check_result(const duo_result* out) {
    if (!out || !out->accept_len || !out->next_token || !out->commit || !out->status) return DUO_ERR_NULL;
    return DUO_OK;
}

constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[NOALLOC_MAX_DEVICES];  // per device: address of that device's copy of `scratch`; nullptr until asked for

// The current device's copy of `scratch`; the first call on a device asks the runtime for its address.
int scratch_of_current_device(void** out) {
    int dev = -1;
    int rc = hip_ok(hipGetDevice(&dev), "hipGetDevice");
    if (rc) return rc;
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) {
        snprintf(g_hip_err, sizeof g_hip_err, "device index %d beyond the %d this library keeps scratch addresses for", dev, NOALLOC_MAX_DEVICES);
        return DUO_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        rc = hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (rc) return rc;
        if (!p) {
            snprintf(g_hip_err, sizeof g_hip_err, "hipGetSymbolAddress(scratch) returned a null address");
            return DUO_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DUO_OK;
}

// duo_spec_sample's sampling kernels on the static scratch array
int spec_sample_on_scratch(const float* logits, const float* root_logits, int vocab, const int32_t* draft_tokens,
                                  const float* draft_probs, const float* uniforms, const duo_call* call, duo_result* out,
                                  void* hip_stream) {
    if (vocab < 2) return DUO_ERR_SHAPE;
    int rc = check_call(call, vocab);
    if (rc) return rc;
    if ((rc = check_result(out))) return rc;
    const int R = call->root_token >= 0 ? 1 : 0;
    if (!logits || !draft_tokens || !draft_probs || !uniforms || (!R && !root_logits)) return DUO_ERR_NULL;
    if (vocab > DUO_NOALLOC_MAX_VOCAB || nucleus_on(call)) return DUO_ERR_SCRATCH;
    void* base = nullptr;
    if ((rc = scratch_of_current_device(&base))) return rc;
    Workspace ws{};
    char* b = static_cast<char*>(base);
    ws.stats_parts = STATS_SPLIT;
    ws.stats_rows = reinterpret_cast<double*>(b);
    ws.stats_root = ws.stats_rows + (size_t)(DUO_MAX_ROWS + 1) * STATS_SPLIT * 2;
    ws.p_run = reinterpret_cast<double*>(b + NOALLOC_STATS_BYTES);
    ws.acc = reinterpret_cast<int32_t*>(b + NOALLOC_STATS_BYTES + NOALLOC_PRUN_BYTES);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    DUO_LAUNCH(fill_i32_kernel, dim3(1), dim3(64), s, out->status, 1, 0);
    SampleArgs sa{logits, vocab, root_logits, vocab, call->n, call->k, R, call->host_prefix_len, (double)call->temperature,
                  draft_tokens, draft_probs, uniforms, ws.stats_rows, ws.stats_parts, ws.stats_root, STATS_SPLIT, ws.acc, ws.p_run, out->accept_len, out->next_token,
                  out->commit, out->status, nullptr};
    enqueue_sampling(sa, call->top_p, ws, call->select_mode, nullptr, nullptr, nullptr, nullptr, s);
    return hip_ok(hipGetLastError(), "duo_spec_sample_noalloc launch");
}

}  // namespace

extern "C" {

int duo_workspace_bytes(const duo_model_config* cfg, int max_rows, size_t* bytes) {
    if (!bytes) return DUO_ERR_NULL;
    int rc = check_config(cfg);
    if (rc) return rc;
    if (max_rows < 1 || max_rows > DUO_MAX_PREFILL_ROWS) return DUO_ERR_SHAPE;
    *bytes = carve(*cfg, max_rows, nullptr).total;
    return DUO_OK;
}

int duo_verify(const duo_model_config* cfg, const duo_weights* w, duo_kv_cache* cache, const int32_t* draft_tokens,
               const float* draft_probs, const float* uniforms, const duo_call* call, duo_result* out, void* workspace,
               size_t workspace_bytes, void* hip_stream) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if ((rc = check_weights(cfg, w))) return rc;
    if (!cache || !cache->k || !cache->v || !cache->prefix_len || !draft_tokens || !draft_probs || !uniforms || !workspace)
        return DUO_ERR_NULL;
    if ((rc = check_call(call, cfg->vocab))) return rc;
    if ((rc = check_result(out))) return rc;
    const int R = call->root_token >= 0 ? 1 : 0;
    if (!R && !cache->root_logits) return DUO_ERR_NULL;
    const int M = R + call->n * call->k;
    if ((long long)call->host_prefix_len + M > cfg->max_seq) return DUO_ERR_CAPACITY;
    if (!aligned16(cache->k) || !aligned16(cache->v) || !aligned16(workspace) || !aligned16(draft_probs) ||
        (out->logits_out && !aligned16(out->logits_out)))
        return DUO_ERR_ALIGN;
    const Workspace ws = carve(*cfg, M, workspace);
    if (workspace_bytes < ws.total) return DUO_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    const RowPlan plan{call->host_prefix_len, R, call->n, call->k, M};  // the pass's first kernel clears *status
    float* logits = out->logits_out ? out->logits_out : ws.logits;
    enqueue_forward(*cfg, *w, *cache, draft_tokens, call->root_token, plan, ws, logits, out->status, s, (double)call->temperature);
    SampleArgs sa{logits, cfg->vocab, cache->root_logits, cfg->vocab, call->n, call->k, R, call->host_prefix_len,
                  (double)call->temperature, draft_tokens, draft_probs, uniforms, ws.stats_rows, ws.stats_parts, ws.stats_root, ROOT_STATS_PARTS, ws.acc, ws.p_run,
                  out->accept_len, out->next_token, out->commit, out->status,
                  nucleus_on(call) ? ws.nuc : nullptr};
    enqueue_sampling(sa, call->top_p, ws, call->select_mode, cache->k, cache->v, cfg, cache->prefix_len, s, true);
    return hip_ok(hipGetLastError(), "duo_verify launch");
}

int duo_prefill_chunk(const duo_model_config* cfg, const duo_weights* w, duo_kv_cache* cache, const int32_t* tokens, int m,
                      int host_prefix_len, int32_t* status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if ((rc = check_weights(cfg, w))) return rc;
    if (!cache || !cache->k || !cache->v || !cache->prefix_len || !cache->root_logits || !tokens || !status || !workspace)
        return DUO_ERR_NULL;
    if (m < 1 || m > DUO_MAX_PREFILL_ROWS) return DUO_ERR_SHAPE;
    if (host_prefix_len < 0) return DUO_ERR_ARG;
    if ((long long)host_prefix_len + m > cfg->max_seq) return DUO_ERR_CAPACITY;
    if (!aligned16(cache->k) || !aligned16(cache->v) || !aligned16(workspace)) return DUO_ERR_ALIGN;
    const Workspace ws = carve(*cfg, m, workspace);
    if (workspace_bytes < ws.total) return DUO_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    const RowPlan plan{host_prefix_len, 0, 1, m, m};  // the pass's first kernel clears *status
    enqueue_forward(*cfg, *w, *cache, tokens, -1, plan, ws, ws.logits, status, s);
    DUO_LAUNCH(prefill_finish_kernel, dim3((cfg->vocab + 255) / 256), dim3(256), s,
                       ws.logits + (m > DUO_MAX_ROWS ? 0 : (size_t)(m - 1) * cfg->vocab), cache->root_logits, cfg->vocab, cache->prefix_len,
                       host_prefix_len + m, status);
    return hip_ok(hipGetLastError(), "duo_prefill_chunk launch");
}

int duo_sample_workspace_bytes(int vocab, int n, int k, size_t* bytes) {
    if (!bytes) return DUO_ERR_NULL;
    if (vocab < 2 || n < 1 || k < 0 || (long long)n * k + 1 > DUO_MAX_ROWS + 1) return DUO_ERR_SHAPE;
    *bytes = sample_ws_bytes(vocab);
    return DUO_OK;
}

int duo_spec_sample(const float* logits, const float* root_logits, int vocab, const int32_t* draft_tokens,
                    const float* draft_probs, const float* uniforms, const duo_call* call, duo_result* out, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
    if (vocab < 2) return DUO_ERR_SHAPE;
    int rc = check_call(call, vocab);
    if (rc) return rc;
    if ((rc = check_result(out))) return rc;
    const int R = call->root_token >= 0 ? 1 : 0;
    if (!logits || !draft_tokens || !draft_probs || !uniforms || !workspace || (!R && !root_logits)) return DUO_ERR_NULL;
    if (!aligned16(workspace)) return DUO_ERR_ALIGN;
    if (workspace_bytes < sample_ws_bytes(vocab)) return DUO_ERR_WORKSPACE;
    Workspace ws{};
    size_t off = 0;
    carve_sampler(static_cast<char*>(workspace), off, vocab, ws);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    DUO_LAUNCH(fill_i32_kernel, dim3(1), dim3(64), s, out->status, 1, 0);
    SampleArgs sa{logits, vocab, root_logits, vocab, call->n, call->k, R, call->host_prefix_len, (double)call->temperature,
                  draft_tokens, draft_probs, uniforms, ws.stats_rows, ws.stats_parts, ws.stats_root, STATS_SPLIT, ws.acc, ws.p_run, out->accept_len, out->next_token,
                  out->commit, out->status,
                  nucleus_on(call) ? ws.nuc : nullptr};
    enqueue_sampling(sa, call->top_p, ws, call->select_mode, nullptr, nullptr, nullptr, nullptr, s);
    return hip_ok(hipGetLastError(), "duo_spec_sample launch");
}

int duo_spec_sample_noalloc(const float* logits, const float* root_logits, int vocab, const int32_t* draft_tokens,
                            const float* draft_probs, const float* uniforms, const duo_call* call, duo_result* out,
                            void* hip_stream) {
    return spec_sample_on_scratch(logits, root_logits, vocab, draft_tokens, draft_probs, uniforms, call, out, hip_stream);
}

// checks shared by the two deferred entry points
static int check_deferred(const duo_call* call, int vocab, const int32_t* first_tokens, const float* first_probs,
                          const float* uniforms_first, int s) {
    int rc = check_call(call, vocab, 0);
    if (rc) return rc;
    if (call->n != 1) return DUO_ERR_SHAPE;
    if (s < 0 || s > DUO_MAX_ROWS) return DUO_ERR_SHAPE;
    if (s > 0 && (!first_tokens || !first_probs || !uniforms_first)) return DUO_ERR_NULL;
    return DUO_OK;
}

static void enqueue_deferred_sampling(const SampleArgs& sa, float top_p, const Workspace& ws, const DeferredArgs& da,
                                      hipStream_t s, bool have_stats = false) {
    if (!have_stats) {
        prof(DUO_PROF_SAMPLE, s);
        DUO_LAUNCH(sample_stats_kernel, dim3(sa.R + sa.k + (sa.R ? 0 : 1), STATS_SPLIT), dim3(256), s, sa);
    }
    enqueue_nucleus(sa, top_p, ws, s);
    prof(DUO_PROF_SAMPLE, s);
    if (sa.nuc) DUO_LAUNCH(sample_deferred_kernel<true>, dim3(1), dim3(SAMPLE_THREADS), s, sa, da);
    else DUO_LAUNCH(sample_deferred_kernel<false>, dim3(1), dim3(SAMPLE_THREADS), s, sa, da);
}

int duo_verify_deferred(const duo_model_config* cfg, const duo_weights* w, duo_kv_cache* cache,
                        const int32_t* unverified_tokens, const float* unverified_probs, const float* uniforms,
                        const int32_t* first_tokens, const float* first_probs, const float* uniforms_first, int s_new,
                        const duo_call* call, duo_result* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if ((rc = check_weights(cfg, w))) return rc;
    if (!cache || !cache->k || !cache->v || !cache->prefix_len || !uniforms || !workspace) return DUO_ERR_NULL;
    if ((rc = check_deferred(call, cfg->vocab, first_tokens, first_probs, uniforms_first, s_new))) return rc;
    if (call->k > 0 && (!unverified_tokens || !unverified_probs)) return DUO_ERR_NULL;  // an empty suffix needs neither
    if ((rc = check_result(out))) return rc;
    const int R = call->root_token >= 0 ? 1 : 0;
    if (!R && !cache->root_logits) return DUO_ERR_NULL;
    const int M = R + call->k;
    if ((long long)call->host_prefix_len + M > cfg->max_seq) return DUO_ERR_CAPACITY;
    if (!aligned16(cache->k) || !aligned16(cache->v) || !aligned16(workspace) || !aligned16(unverified_probs) ||
        (out->logits_out && !aligned16(out->logits_out)))
        return DUO_ERR_ALIGN;
    const Workspace ws = carve(*cfg, M > 0 ? M : 1, workspace);
    if (workspace_bytes < ws.total) return DUO_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    float* logits = out->logits_out ? out->logits_out : ws.logits;
    if (M > 0) {
        // an empty suffix leaves the root token as the pass's only row (the plan's k is then never used as a divisor)
        const RowPlan plan{call->host_prefix_len, R, 1, call->k > 0 ? call->k : 1, M};  // the pass's first kernel clears *status
        enqueue_forward(*cfg, *w, *cache, unverified_tokens, call->root_token, plan, ws, logits, out->status, s, (double)call->temperature);
    } else {
        // nothing to score: the cached root logits judge the new sequences; only the device-side input check runs
        DUO_LAUNCH(status_init_kernel, dim3(1), dim3(64), s, out->status, cache->prefix_len, call->host_prefix_len);
    }
    SampleArgs sa{logits, cfg->vocab, cache->root_logits, cfg->vocab, 1, call->k, R, call->host_prefix_len,
                  (double)call->temperature, unverified_tokens, unverified_probs, uniforms, ws.stats_rows, ws.stats_parts, ws.stats_root, M > 0 ? ROOT_STATS_PARTS : STATS_SPLIT, ws.acc, ws.p_run,
                  out->accept_len, out->next_token, out->commit, out->status,
                  nucleus_on(call) ? ws.nuc : nullptr};
    enqueue_deferred_sampling(sa, call->top_p, ws, DeferredArgs{first_tokens, first_probs, uniforms_first, s_new, cache->prefix_len}, s,
                              M > 0);  // a pass that scored rows left their statistics and the root logits'
    return hip_ok(hipGetLastError(), "duo_verify_deferred launch");
}

int duo_deferred_sample(const float* logits, const float* root_logits, int vocab, const int32_t* unverified_tokens,
                        const float* unverified_probs, const float* uniforms, const int32_t* first_tokens,
                        const float* first_probs, const float* uniforms_first, int s_new, const duo_call* call,
                        duo_result* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (vocab < 2) return DUO_ERR_SHAPE;
    int rc = check_deferred(call, vocab, first_tokens, first_probs, uniforms_first, s_new);
    if (rc) return rc;
    if ((rc = check_result(out))) return rc;
    const int R = call->root_token >= 0 ? 1 : 0;
    if (!uniforms || !workspace || (!R && !root_logits) || (R + call->k > 0 && !logits)) return DUO_ERR_NULL;
    if (call->k > 0 && (!unverified_tokens || !unverified_probs)) return DUO_ERR_NULL;
    if (!aligned16(workspace)) return DUO_ERR_ALIGN;
    if (workspace_bytes < sample_ws_bytes(vocab)) return DUO_ERR_WORKSPACE;
    Workspace ws{};
    size_t off = 0;
    carve_sampler(static_cast<char*>(workspace), off, vocab, ws);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    DUO_LAUNCH(fill_i32_kernel, dim3(1), dim3(64), s, out->status, 1, 0);
    SampleArgs sa{logits, vocab, root_logits, vocab, 1, call->k, R, call->host_prefix_len, (double)call->temperature,
                  unverified_tokens, unverified_probs, uniforms, ws.stats_rows, ws.stats_parts, ws.stats_root, STATS_SPLIT, ws.acc, ws.p_run, out->accept_len, out->next_token,
                  out->commit, out->status,
                  nucleus_on(call) ? ws.nuc : nullptr};
    enqueue_deferred_sampling(sa, call->top_p, ws, DeferredArgs{first_tokens, first_probs, uniforms_first, s_new, nullptr}, s);
    return hip_ok(hipGetLastError(), "duo_deferred_sample launch");
}

int duo_skinny_gemm(const uint16_t* x, const uint16_t* w, float* y, int rows, int N, int K, void* hip_stream) {
    if (!x || !w || !y) return DUO_ERR_NULL;
    if (rows < 1 || rows > DUO_MAX_ROWS || N < 1 || K < 32 || K % 32) return DUO_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(w)) return DUO_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    EpiStoreF32 e{N, rows, 2, y, N};
    launch_gemm_rows<2>(rows, false, x, w, K, (N + 31) / 32, RowScale{nullptr, 0, 0.f, 0.f, nullptr}, e, s);
    return hip_ok(hipGetLastError(), "duo_skinny_gemm launch");
}

int duo_block_gemm(const uint16_t* x, const uint16_t* w, float* y, int rows, int N, int K, void* hip_stream) {
    if (!x || !w || !y) return DUO_ERR_NULL;
    if (rows < 1 || rows > DUO_MAX_PREFILL_ROWS || N < 1 || K < 32 || K % 32) return DUO_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(w)) return DUO_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    EpiStoreF32 e{N, rows, 1, y, N, 0};
    launch_block<4, 4, 1>(x, w, K, (N + 15) / 16, rows, 1, RowScale{nullptr, 0, 0.f, 0.f, nullptr}, e, s);
    return hip_ok(hipGetLastError(), "duo_block_gemm launch");
}

int duo_stream_read_probe(const void* src, size_t bytes, uint32_t* sink, int sink_len, int nontemporal, void* hip_stream) {
    if (!src || !sink) return DUO_ERR_NULL;
    if (bytes < 16 || sink_len < 1) return DUO_ERR_SHAPE;
    if (!aligned16(src)) return DUO_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    const int grid = sink_len < 2048 ? sink_len : 2048;
    if (nontemporal) DUO_LAUNCH(stream_read_kernel<true>, dim3(grid), dim3(256), s, static_cast<const u32x4*>(src), bytes / 16, sink);
    else DUO_LAUNCH(stream_read_kernel<false>, dim3(grid), dim3(256), s, static_cast<const u32x4*>(src), bytes / 16, sink);
    return hip_ok(hipGetLastError(), "duo_stream_read_probe launch");
}

size_t duo_k_cache_offset(int head_dim, int slot, int channel) { return k_cache_offset(head_dim, slot, channel); }
size_t duo_v_cache_offset(int head_dim, int slot, int channel) { return v_cache_offset(head_dim, slot, channel); }

size_t duo_packed_elems(int N, int K) {
    if (N < 1 || K < 1) return 0;
    return (size_t)((N + 31) / 32) * 32 * (size_t)K;
}

int duo_pack_matrix(const uint16_t* src, int N, int K, uint16_t* dst, void* hip_stream) {
    if (!src || !dst) return DUO_ERR_NULL;
    if (N < 1 || K < 32 || K % 32) return DUO_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return DUO_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    DUO_LAUNCH((pack_bands_kernel<PlainRows>), dim3((N + 31) / 32 * 2), dim3(256), s, PlainRows{src, N, K}, K / 32,
                       dst);
    return hip_ok(hipGetLastError(), "duo_pack_matrix launch");
}

int duo_pack_qkv(const duo_model_config* cfg, const uint16_t* wq, const uint16_t* wk, const uint16_t* wv, uint16_t* dst,
                 void* hip_stream) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!wq || !wk || !wv || !dst) return DUO_ERR_NULL;
    if (!aligned16(wq) || !aligned16(wk) || !aligned16(wv) || !aligned16(dst)) return DUO_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    const int D = cfg->head_dim, half = D / 2, bph = D / 16;
    const int bands = (cfg->n_q_heads + 2 * cfg->n_kv_heads) * bph;
    DUO_LAUNCH((pack_bands_kernel<QKVRows>), dim3(bands), dim3(256), s,
                       QKVRows{wq, wk, wv, cfg->n_q_heads, cfg->n_kv_heads, D, half, bph, cfg->d_model}, cfg->d_model / 32, dst);
    return hip_ok(hipGetLastError(), "duo_pack_qkv launch");
}

int duo_pack_gate_up(const duo_model_config* cfg, const uint16_t* w_gate, const uint16_t* w_up, uint16_t* dst,
                     void* hip_stream) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!w_gate || !w_up || !dst) return DUO_ERR_NULL;
    if (!aligned16(w_gate) || !aligned16(w_up) || !aligned16(dst)) return DUO_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    DUO_LAUNCH((pack_bands_kernel<GateUpRows>), dim3(cfg->d_ff / 16 * 2), dim3(256), s,
                       GateUpRows{w_gate, w_up, cfg->d_ff, cfg->d_model}, cfg->d_model / 32, dst);
    return hip_ok(hipGetLastError(), "duo_pack_gate_up launch");
}

int duo_pack_activations(const uint16_t* src, int rows, int K, uint16_t* dst, void* hip_stream) {
    if (!src || !dst) return DUO_ERR_NULL;
    if (rows < 1 || rows > 2 * DUO_MAX_PREFILL_ROWS || K < 32 || K % 32) return DUO_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return DUO_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    DUO_LAUNCH(pack_operand_kernel, dim3(K / 32), dim3(256), s, src, rows, K, (rows + 15) / 16, dst);
    return hip_ok(hipGetLastError(), "duo_pack_activations launch");
}

int duo_profile_enable(int enable) {
    if (enable && g_prof.ev.empty()) {
        g_prof.ev.resize(2 * PROF_POOL);
        g_prof.cls.assign(PROF_POOL, -1);
        for (auto& e : g_prof.ev) {
            int rc = hip_ok(hipEventCreate(&e), "hipEventCreate");
            if (rc) return rc;
        }
    }
    g_prof.on = enable != 0;
    g_prof.used = 0;
    g_prof.dropped = 0;
    g_launch_events = LaunchEvents{};
    return DUO_OK;
}

int duo_profile_dropped(void) { return (int)g_prof.dropped; }

const char* duo_profile_kernel_name(int cls) { return (cls >= 0 && cls < DUO_PROF_CLASSES) ? g_prof.names[cls] : ""; }

int duo_profile_read(double* ms, int32_t* launches) {
    if (!ms || !launches) return DUO_ERR_NULL;
    for (int i = 0; i < DUO_PROF_CLASSES; ++i) {
        ms[i] = 0.0;
        launches[i] = 0;
    }
    for (size_t i = 0; i < g_prof.used; ++i) {
        int rc = hip_ok(hipEventSynchronize(g_prof.ev[2 * i + 1]), "hipEventSynchronize");
        if (rc) return rc;
        float t = 0.f;
        if ((rc = hip_ok(hipEventElapsedTime(&t, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]), "hipEventElapsedTime"))) return rc;
        ms[g_prof.cls[i]] += t;
        launches[g_prof.cls[i]] += 1;
    }
    g_prof.used = 0;
    g_prof.dropped = 0;
    return DUO_OK;
}

const char* duo_status_string(int code) {
    switch (code) {
        case DUO_OK: return "ok";
        case DUO_ERR_NULL: return "required pointer is NULL";
        case DUO_ERR_SHAPE: return "unsupported shape";
        case DUO_ERR_CAPACITY: return "KV cache capacity exceeded";
        case DUO_ERR_ALIGN: return "pointer not 16-byte aligned";
        case DUO_ERR_WORKSPACE: return "workspace too small";
        case DUO_ERR_TOKEN_RANGE: return "token id out of range";
        case DUO_ERR_HIP: return "HIP error";
        case DUO_ERR_ARG: return "invalid argument";
        case DUO_ERR_SCRATCH: return "request exceeds the static scratch of the no-allocation entry point (vocabulary above DUO_NOALLOC_MAX_VOCAB, or top_p)";
        default: return "unknown status";
    }
}

const char* duo_last_hip_error(void) { return g_hip_err; }

}  // extern "C"
