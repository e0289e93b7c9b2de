/*
 * duo_verify.h -- C ABI of the MI355X (gfx950) target-side verification step of DuoDecoding
 * (arxiv 2503.00784).
 *
 * One call scores n draft sequences of k tokens with the target model in a single forward
 * pass (Alg. 1, right column: p <- M_p(x); Sec. 1: all candidates are scored by one pass of the
 * target), the sequences being independent branches of a shared prefix (Sec. 3.2,
 * Fig. 2), then verifies them by speculative sampling (Alg. 2, Sec. 3.3) and commits the
 * accepted tokens' keys and values to the cache.  The draft model, the draft budget and the
 * CPU/GPU scheduling of Alg. 1 are host work and not part of this library: draft tokens,
 * draft distributions and the uniform random numbers of Alg. 2 are inputs.
 *
 * Conventions
 *   - Every pointer below is a DEVICE pointer unless it is marked HOST.  The library never
 *     allocates, frees or keeps caller memory; scratch space is the caller's `workspace`.
 *   - All work is enqueued on `hip_stream` (a hipStream_t cast to void*; NULL = default
 *     stream) without host synchronisation.  Arguments are validated on the host before
 *     anything is enqueued; a negative return code means nothing was enqueued.
 *   - 16-bit values (weights, gains, embedding, KV cache) are passed as uint16_t bit patterns.  The library is
 *     built twice from the same sources with the same entry points: libduo_verify.so takes them as bf16
 *     (wherever this header says bf16), libduo_verify_fp16.so as IEEE fp16, the precision the paper ran its
 *     target model in (Sec. 4.1).  A process may load both.  Matrices compute y = x W^T, are 16-byte
 *     aligned, and have an input dimension that is a multiple of 32.
 *   - A call with the same inputs and the same `host_prefix_len` is repeatable: cache slots
 *     below the prefix length are only read, slots at and above it are scratch.
 */
#ifndef DUO_VERIFY_H
#define DUO_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DUO_OK               0
#define DUO_ERR_NULL        -1  /* a required pointer is NULL */
#define DUO_ERR_SHAPE       -2  /* unsupported model geometry or n, k out of range */
#define DUO_ERR_CAPACITY    -3  /* prefix + rows of this call exceed max_seq */
#define DUO_ERR_ALIGN       -4  /* a pointer is not 16-byte aligned */
#define DUO_ERR_WORKSPACE   -5  /* workspace smaller than duo_workspace_bytes() */
#define DUO_ERR_TOKEN_RANGE -6  /* root_token >= vocab */
#define DUO_ERR_HIP         -7  /* a HIP call failed; see duo_last_hip_error() */
#define DUO_ERR_ARG         -8  /* temperature < 0 or NaN, unknown select_mode, ... */
#define DUO_ERR_SCRATCH     -9  /* duo_spec_sample_noalloc: vocabulary above DUO_NOALLOC_MAX_VOCAB, or top_p asked for */

/* Most rows one call can score: n*k (+1 with a root token). */
#define DUO_MAX_ROWS 80
#define DUO_MAX_PREFILL_ROWS 1024 /* rows of one duo_prefill_chunk call */

/* Bits of the device-side status word (duo_result.status), set by kernels that cannot be
 * checked on the host without a synchronisation.  A call whose status word is not clean FAILED ON THE DEVICE and
 * commits nothing: *cache.prefix_len and every cache slot below it are left exactly as they were (on a prefix
 * mismatch the pass writes no keys or values at all; slots at and above the device's prefix length are scratch in any
 * case), root_logits is not replaced by duo_prefill_chunk, and the commit record reads
 * {-1, 0, -1, unchanged prefix length}.  accept_len / next_token / logits_out then hold no usable result. */
#define DUO_STATUS_TOKEN_CLAMPED   1  /* a draft token id was outside [0, vocab) and was clamped */
#define DUO_STATUS_PREFIX_MISMATCH 2  /* *cache.prefix_len differed from call.host_prefix_len */

#define DUO_SELECT_INDEPENDENT_LONGEST 0
#define DUO_SELECT_PAPER_SEQUENTIAL    1

/* Geometry of the Llama-shaped target (the architecture of the paper's targets, Sec. 4.1
 * "Models").  head_dim is 64 or 128; d_model is a multiple of 64 (at most 8192), n_q_heads*head_dim and d_ff
 * are multiples of 32; n_q_heads is a multiple of n_kv_heads; max_seq is a multiple of 32. */
typedef struct duo_model_config {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab, max_seq;
    float   rope_theta; /* rotary base; pair (d, d + head_dim/2) turns by pos * theta^(-2d/head_dim) */
    float   rms_eps;
} duo_model_config;

/*
 * Parameters, bf16.  Every matrix the step streams is held in the library's STREAMING LAYOUT, made
 * once at load time by the duo_pack_* calls below from ordinary row-major [out][in] matrices: bands
 * of 16 output rows, cut into 16 x 32 tiles of 1 KiB that are contiguous and ordered the way one MFMA
 * operand sits in a wavefront's registers, so that a wave reads its band as one linear stream.  The
 * embedding table is gathered, not streamed, and stays row-major.  The seven per-layer tables are
 * HOST arrays of n_layers DEVICE pointers.
 */
typedef struct duo_weights {
    const uint16_t *embed;                    /* row-major [vocab][d_model] */
    const uint16_t *const *wqkv;              /* duo_pack_qkv of wq [n_q_heads*head_dim][d_model] and
                                                 wk, wv [n_kv_heads*head_dim][d_model] */
    const uint16_t *const *wo;                /* duo_pack_matrix of [d_model][n_q_heads*head_dim] */
    const uint16_t *const *w_gate_up;         /* duo_pack_gate_up of w_gate, w_up [d_ff][d_model] */
    const uint16_t *const *w_down;            /* duo_pack_matrix of [d_model][d_ff] */
    const uint16_t *const *g_attn, *const *g_ffn; /* RMSNorm gains [d_model] */
    const uint16_t *g_final;                  /* [d_model] */
    const uint16_t *lm_head;                  /* duo_pack_matrix of [vocab][d_model] */
} duo_weights;

/*
 * Repacking into the streaming layout (device to device, enqueued on the stream, done once per
 * model).  src matrices are row-major bf16, 16-byte aligned, K a multiple of 32.  dst needs
 * duo_packed_elems(N, K) uint16 elements: N is rounded up to a multiple of 32 rows, missing rows are
 * zero.  duo_pack_qkv needs duo_packed_elems((n_q_heads + 2*n_kv_heads)*head_dim, d_model) and orders
 * the rows so that every band holds eight channels of a head next to their eight rotary partners;
 * duo_pack_gate_up needs duo_packed_elems(2*d_ff, d_model) and interleaves gate and up bands.
 */
size_t duo_packed_elems(int N, int K);
int duo_pack_matrix(const uint16_t *src, int N, int K, uint16_t *dst, void *hip_stream);
int duo_pack_qkv(const duo_model_config *cfg, const uint16_t *wq, const uint16_t *wk, const uint16_t *wv,
                 uint16_t *dst, void *hip_stream);
int duo_pack_gate_up(const duo_model_config *cfg, const uint16_t *w_gate, const uint16_t *w_up, uint16_t *dst,
                     void *hip_stream);
/* Activation rows [rows][K] (row-major) -> operand layout for duo_skinny_gemm; dst needs
 * ((rows + 15) / 16) * 16 * K elements. */
int duo_pack_activations(const uint16_t *src, int rows, int K, uint16_t *dst, void *hip_stream);

/* KV cache, bf16, caller-owned: k and v each hold n_layers * n_kv_heads planes of max_seq * head_dim
 * elements (plane index layer * n_kv_heads + kv_head).  Inside a plane both are stored as the 1 KiB tiles the
 * attention kernels feed to the matrix cores, 32 slots at a time, so that a wavefront fetches a tile with one
 * fully coalesced load.  Keys are stored after the rotary embedding.  With D = head_dim, block B = slot / 32
 * and w = slot % 32, the element (slot, channel d) of a plane is at
 *   K: ((((B*2 + t) * (D/32) + d/32) * 64 + ((d%32)/8) * 16 + 4*(w/8) + w%4) * 8 + d%8,  t = (w%8)/4
 *   V: (((B * (D/16) + d/16) * 64 + (w/8) * 16 + d%16) * 8 + w%8
 * (V is in effect transposed: a lane's eight consecutive elements are eight consecutive slots of one channel).
 * duo_k_cache_offset / duo_v_cache_offset evaluate these on the host.  Slots [0, *prefix_len) hold the shared
 * prefix. */
size_t duo_k_cache_offset(int head_dim, int slot, int channel);
size_t duo_v_cache_offset(int head_dim, int slot, int channel);

typedef struct duo_kv_cache {
    uint16_t *k;
    uint16_t *v;
    int32_t  *prefix_len;   /* device scalar P; advanced by the commit */
    float    *root_logits;  /* fp32 [vocab]: target logits after the last prefix token (from
                               prefill); read when root_token < 0, may be NULL otherwise */
} duo_kv_cache;

typedef struct duo_call {
    int32_t n, k;            /* n sequences of k draft tokens, n*k + (root?1:0) <= DUO_MAX_ROWS */
    float   temperature;     /* p = softmax(logits / temperature), > 0; exactly 0 = the greedy limit of Alg. 2: p is
                                one-hot at the largest logit (lowest id among equal logits), so a draft token is
                                accepted iff it is that id and every correction / bonus token is that id; the
                                uniforms are still read but cannot change the outcome */
    int32_t select_mode;     /* DUO_SELECT_* */
    int32_t root_token;      /* >= 0: the token emitted by the previous step, scored as one shared
                                row in front of every sequence (its logits judge the first draft
                                tokens); < 0: cache.root_logits judges them */
    int32_t host_prefix_len; /* P as the host knows it; sizes the launch and is checked on device */
    float   top_p;           /* 0 < top_p < 1 (and temperature > 0): every target distribution is first restricted to its
                                nucleus, the most probable tokens in order of decreasing probability (equal ones by
                                ascending id) up to and including the one with which their mass reaches top_p, and
                                renormalised; Alg. 2 then runs on the restricted distributions.  Any other value
                                (0 included): no restriction.  The draft distributions are taken as given. */
} duo_call;

/* Outputs (device).  Alg. 2 returns the new prefix length, the new prefix and the unverified
 * suffix; here: per-sequence accepted lengths, the correction / bonus token, and the commit. */
typedef struct duo_result {
    int32_t *accept_len; /* [n]  leading accepted draft tokens of each sequence; in paper mode 0 for
                                 sequences rejected before the selected one, -1 for those after it */
    int32_t *next_token; /* [n]  correction token (residual sample at the first rejection) or bonus
                                 token (all k accepted); paper mode: only the selected entry, else -1 */
    int32_t *commit;     /* [4]  {selected sequence or -1, commit_len, commit_token, new prefix length} */
    int32_t *status;     /* [1]  DUO_STATUS_* bits, 0 when clean */
    float   *logits_out; /* optional fp32 [rows][vocab] (rows = (root?1:0) + n*k), may be NULL */
} duo_result;

/* Bytes of device scratch a call of up to `max_rows` rows needs: duo_verify takes at most DUO_MAX_ROWS rows,
 * duo_prefill_chunk at most DUO_MAX_PREFILL_ROWS.  Not monotonic across DUO_MAX_ROWS (a pass of more rows keeps the
 * logits of its last row only): a caller that makes both kinds of call allocates the larger of
 * duo_workspace_bytes(DUO_MAX_ROWS) and duo_workspace_bytes(its largest prefill chunk). */
int duo_workspace_bytes(const duo_model_config *cfg, int max_rows, size_t *bytes);

/*
 * The whole step.  Rows: the root token (if any) at position P and cache slot P, draft token
 * (i, j) at position P + R + j and slot P + R + i*k + j (R = 1 with a root token).  Row (i, j)
 * attends to the prefix, the root and (i, j' <= j).  logits of row (i, j) score the token after
 * draft (i, j): draft (i, 0) is judged by the root distribution, draft (i, j >= 1) by row
 * (i, j-1), the bonus token is drawn from row (i, k-1).
 *
 * Speculative sampling (Alg. 2; accept iff u * q(t) < p(t), i.e. with probability
 * min(1, p/q); on rejection sample norm(max(0, p - q)) by inverse CDF over ascending ids):
 *   INDEPENDENT_LONGEST  every sequence is verified on its own, token by token, as one sequence is in plain
 *                        speculative sampling (Sec. 3.3); the longest (lowest index on ties) is committed.
 *   PAPER_SEQUENTIAL     first tokens are tested in order against the root distribution, which
 *                        is replaced by its normalised residual after each rejection (Alg. 2,
 *                        multi-sequence block); the first accepted sequence is verified to its
 *                        end; if none is accepted a token is drawn from the final residual.
 * uniforms[i][j] (j < k) tests draft (i, j); uniforms[i][k] drives the correction / bonus sample
 * (paper mode, none accepted: uniforms[n-1][k]).
 *
 * Commit: keys/values of the selected sequence's first commit_len tokens are moved to slots
 * P + R + 0.., *prefix_len becomes P + R + commit_len.  The emitted token is not in the cache;
 * pass it as root_token to the next call.
 *
 * draft_tokens int32 [n][k]; draft_probs fp32 [n][k][vocab] (full draft distributions, needed
 * for residuals); uniforms fp32 [n][k+1] in [0, 1).
 */
int duo_verify(const duo_model_config *cfg, const duo_weights *w, duo_kv_cache *cache,
               const int32_t *draft_tokens, const float *draft_probs, const float *uniforms,
               const duo_call *call, duo_result *out,
               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Scores m <= DUO_MAX_PREFILL_ROWS tokens (device int32) as a continuation of the cached prefix with a
 * plain causal mask, appends their keys/values, advances *prefix_len by m and stores the last
 * row's logits in cache->root_logits: the target pass of Alg. 1 applied to prompt tokens (the target model's
 * share of the time to first token, Sec. 4.1).  Up to DUO_MAX_ROWS rows run through the verify pass's
 * weight-streaming kernels; more rows through projection kernels that stage both operands in LDS, and only
 * the last row's logits are computed.  `workspace` needs duo_workspace_bytes(cfg, m) bytes.
 */
int duo_prefill_chunk(const duo_model_config *cfg, const duo_weights *w, duo_kv_cache *cache,
                      const int32_t *tokens, int m, int host_prefix_len, int32_t *status,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Speculative sampling alone (the second half of duo_verify) on logits the caller supplies:
 * logits fp32 [R + n*k][vocab] with row stride `vocab`.  Does not touch any KV cache; writes
 * accept_len, next_token and commit as duo_verify does (new prefix length = host_prefix_len +
 * R + commit_len).  `workspace` needs duo_sample_workspace_bytes(vocab, n, k) bytes.
 */
int duo_sample_workspace_bytes(int vocab, int n, int k, size_t *bytes);
int duo_spec_sample(const float *logits, const float *root_logits, int vocab,
                    const int32_t *draft_tokens, const float *draft_probs, const float *uniforms,
                    const duo_call *call, duo_result *out,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * duo_spec_sample for callers that cannot allocate or pass a workspace (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same sampling kernels, with their scratch (softmax statistics, accept
 * flags, one running distribution) in a static device array of DUO_NOALLOC_SCRATCH_BYTES inside the library, which
 * every device the library runs on holds until the process ends.  Same arguments and results as duo_spec_sample
 * without the workspace.  Limits: vocab <= DUO_NOALLOC_MAX_VOCAB and no nucleus restriction (0 < top_p < 1 at a
 * positive temperature), else DUO_ERR_SCRATCH and nothing is enqueued.  Calls no hipMalloc / hipFree and no
 * allocating routine.  The first call on a device (with that device current, as for every call) asks the runtime
 * for the address of that device's copy of the array; make it outside a stream capture.  All calls on one device
 * share the array: calls that overlap on one device (different streams) race, calls on one stream do not.  Nothing
 * in the array needs clearing between calls: every entry a call reads it has written first.
 */
#define DUO_NOALLOC_MAX_VOCAB 131072
#define DUO_NOALLOC_SCRATCH_BYTES (20480 + 131072 * 8 + 512)
int duo_spec_sample_noalloc(const float *logits, const float *root_logits, int vocab,
                            const int32_t *draft_tokens, const float *draft_probs, const float *uniforms,
                            const duo_call *call, duo_result *out, void *hip_stream);

/*
 * Alg. 2 in the form the paper lists it, for one round of the pipelined loop of Alg. 1: the pass
 * scores the l tokens that the previous round appended without verifying them (the unverified
 * suffix), then
 *   - verifies them in order (accept token m iff u_m * q_m(t) < p_m(t)); at the first rejection the
 *     token is replaced by a draw from norm(max(0, p_m - q_m)) and everything after it is dropped;
 *   - if all l were accepted, judges ONLY THE FIRST TOKEN of each of s new draft sequences, in index
 *     order, against the target distribution after the last scored token, replacing that
 *     distribution by its normalised residual after every rejection; the first accepted sequence is
 *     taken whole (its first token verified, the rest becoming the next round's unverified suffix);
 *   - if none is accepted, draws one token from the final residual.
 * Inputs (device): unverified_tokens int32 [l]; unverified_probs fp32 [l][vocab] (the draft
 * distributions they were drawn from); uniforms fp32 [l + 1]: u_0 .. u_{l-1} and the uniform of the
 * final draw; first_tokens int32 [s], first_probs fp32 [s][vocab], uniforms_first fp32 [s] (s may be
 * 0: then the pointers may be NULL and the last case applies).  call->n must be 1, call->k = l,
 * call->select_mode must hold a valid value and is otherwise ignored, root_token / host_prefix_len as in
 * duo_verify; s <= DUO_MAX_ROWS.
 * l = 0 is the round after a rejection (Alg. 2 then leaves no unverified suffix) and the first round after the
 * prompt: unverified_tokens / unverified_probs may be NULL, uniforms holds the one uniform of the final draw, and
 * the new sequences are judged by the distribution after the root token (the pass scores that one row), or, with
 * root_token < 0, by cache.root_logits without any forward pass.
 * Outputs: out->accept_len[0] = number of accepted suffix tokens a (0..l); out->commit =
 * {index of the accepted new sequence or -1, a, emitted token or -1 when a sequence was accepted,
 * new prefix length P + R + a}; out->next_token[0] = the emitted token or -1.  The keys/values of
 * the accepted suffix tokens stay where the pass wrote them (slots P + R ..) and *prefix_len becomes
 * P + R + a.  An accepted sequence is not in the cache yet: the next round passes its first token as
 * root_token and the rest as the unverified suffix.
 */
int duo_verify_deferred(const duo_model_config *cfg, const duo_weights *w, duo_kv_cache *cache,
                        const int32_t *unverified_tokens, const float *unverified_probs, const float *uniforms,
                        const int32_t *first_tokens, const float *first_probs, const float *uniforms_first,
                        int s, const duo_call *call, duo_result *out,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The sampling half of duo_verify_deferred on logits the caller supplies (fp32 [R + l][vocab], row
 * stride vocab; root_logits judge the first suffix token when call->root_token < 0).  No KV cache is
 * touched; `workspace` needs duo_sample_workspace_bytes(vocab, 1, l) bytes.
 */
int duo_deferred_sample(const float *logits, const float *root_logits, int vocab,
                        const int32_t *unverified_tokens, const float *unverified_probs, const float *uniforms,
                        const int32_t *first_tokens, const float *first_probs, const float *uniforms_first,
                        int s, const duo_call *call, duo_result *out,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * One skinny weight-streaming product, the building block of the target pass:
 * y[m][n] = sum_k x[m][k] * w[n][k]; x from duo_pack_activations (rows <= DUO_MAX_ROWS), w from
 * duo_pack_matrix (N x K, K % 32 == 0), y fp32 [rows][N] row-major.
 */
int duo_skinny_gemm(const uint16_t *x_packed, const uint16_t *w_packed, float *y, int rows, int N, int K,
                    void *hip_stream);

/*
 * The projection kernel of the many-row (prefill) pass on its own, for tests and kernel benchmarks.  The
 * activations are bf16 pairs a = hi + lo: x_packed comes from duo_pack_activations over 2*PR rows, PR = rows
 * rounded up to a multiple of 16, rows [0, rows) holding the hi parts and rows [PR, PR + rows) the lo parts
 * (all other rows zero).  y[m][n] = sum_k (hi + lo)[m][k] * w[n][k], fp32 [rows][N] row-major; w from
 * duo_pack_matrix; rows <= DUO_MAX_PREFILL_ROWS, K % 32 == 0.  Device pointers.
 */
int duo_block_gemm(const uint16_t *x_packed, const uint16_t *w_packed, float *y, int rows, int N, int K,
                   void *hip_stream);

/*
 * Measurement aid: reads `bytes` (rounded down to a multiple of 16) of device memory once with 16-byte loads (ordinary
 * ones, or with nontemporal != 0 loads that carry the non-temporal hint, as the projection kernels' weight loads do),
 * min(sink_len, 2048) workgroups of 256 lanes, and xors what it read into sink[0 .. min(sink_len, 2048)) (device,
 * uint32, caller-initialised).  Timed over a buffer much larger than the caches it gives the read bandwidth a
 * weight-streaming kernel can reach on the device at hand, next to which the projection kernels' rates are read.
 */
int duo_stream_read_probe(const void *src, size_t bytes, uint32_t *sink, int sink_len, int nontemporal, void *hip_stream);

/*
 * Per-kernel timing for the roofline report (the per-iteration time breakdown of Sec. 4.4
 * "Profiling", at kernel granularity).  While enabled, every kernel that duo_verify /
 * duo_prefill_chunk launch carries a start and a stop HIP event that take the dispatch's own begin and
 * end timestamps; duo_profile_read waits for them, adds each kernel's duration to its class, returns
 * the sums (milliseconds) and launch counts accumulated since the last read, and resets them.
 * Enabling allocates a pool of events, and at most 8192 launches are recorded between two reads (a 64-row step is
 * about 260); duo_profile_dropped returns how many launches since the last read (or enable) found the pool
 * empty and went untimed -- call it before duo_profile_read, which resets it.  A call made while profiling is
 * not allocation-free or capturable.  Not thread-safe.
 * ms and launches are HOST arrays of DUO_PROF_CLASSES entries.
 */
#define DUO_PROF_SETUP     0  /* rotary table, embedding gather + first RMSNorm */
#define DUO_PROF_QKV       1  /* fused QKV projection + rotary + KV scatter */
#define DUO_PROF_ATTN      2  /* masked attention over prefix + drafts (chunk partials) */
#define DUO_PROF_ATTN_COMB 3  /* merge of the chunk partials (long contexts only) */
#define DUO_PROF_OPROJ     4  /* O projection + residual */
#define DUO_PROF_RESID_REDUCE 5 /* more than 16 rows: sum of the K-split O/down partial results + residual */
#define DUO_PROF_GATEUP    6  /* gate/up projection + SwiGLU */
#define DUO_PROF_DOWN      7  /* down projection + residual */
#define DUO_PROF_LMHEAD    8  /* LM head */
#define DUO_PROF_SAMPLE    9  /* softmax statistics, accept tests, correction/bonus sampling */
#define DUO_PROF_COMMIT    10 /* sequence selection + KV commit */
#define DUO_PROF_QKV_FINISH 11 /* 49 rows and more: sum of the K-split Q/K/V partial results + rotary + KV scatter */
#define DUO_PROF_CLASSES   12
int duo_profile_enable(int enable);
int duo_profile_read(double *ms, int32_t *launches);
int duo_profile_dropped(void);
/* Name, with template arguments as a kernel trace prints them, of the projection kernel most recently launched under
 * class `cls` while the timer was enabled ("" if none, or if that class's kernels are not named); HOST string, valid until
 * the next profiled launch of the class.  It lets a timing be matched with profiler counter summaries of that kernel. */
const char *duo_profile_kernel_name(int cls);

const char *duo_status_string(int code);
const char *duo_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DUO_VERIFY_H */
