/*
 * hh.h -- C ABI of the component-aware self-speculative decoding hot path for a
 * parallel-hybrid (Mamba-2 branch + GQA attention branch, summed per block)
 * decoder on one MI355X (gfx950).
 *
 * The calls follow the paper's statement of a speculative round (Section 3.3,
 * "Draft Generation and Verification Protocol"): draft k tokens with the
 * SSM-only subgraph M_S (Section 3.2, Eq. 4: attention output suppressed at
 * every layer), verify them with one pass of the full hybrid M_H (Eq. 2), and
 * under greedy decoding accept the longest prefix on which both argmaxes agree.
 *
 * Conventions
 *  - Every call returns an hh_status and never throws.  Argument and ordering
 *    errors are detected on the host before anything is enqueued and leave all
 *    device state untouched.
 *  - The library allocates no device memory: the caller passes one workspace
 *    (size from hh_workspace_bytes) and the weights, all device pointers, which
 *    must outlive the context.  Weight pointers are borrowed, never written.
 *  - Work calls (prefill, draft, set_drafts, verify, commit) are asynchronous on
 *    the HIP stream given as `void* stream` (a hipStream_t; NULL = default
 *    stream).  All calls of one context must use streams that are ordered with
 *    respect to each other.  Calls on one context are not thread-safe.
 *  - Read-back calls (hh_get_*) synchronise the given stream and copy to HOST
 *    pointers.  They are not part of the hot path.
 *  - Order: create -> prefill -> (draft -> verify -> commit)* ; prefill may be
 *    called again to start a new batch.  Violations return HH_ESTATE.
 *  - Matrices are row-major [out][in] in cfg.w_dtype (float32 or bfloat16).
 *    Vectors (norm weights, conv taps [conv_dim][d_conv], conv bias, a_log,
 *    d_skip, dt_bias) are always float32.  The residual stream, SSM and conv
 *    state, softmax and logits are float32; the KV cache is stored in w_dtype.
 *  - Token ids, lengths and acceptance counts are int32.
 */
#ifndef HH_H
#define HH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HH_API __attribute__((visibility("default")))

typedef struct hh_ctx hh_ctx; /* opaque, host memory owned by the library */

typedef enum {
  HH_OK = 0,
  HH_EINVAL = -1,     /* bad argument or configuration */
  HH_ESTATE = -2,     /* call out of order */
  HH_ECAPACITY = -3,  /* batch, sequence length, draft length or generation budget exceeds capacity */
  HH_EWORKSPACE = -4, /* workspace missing, misaligned or too small */
  HH_EDEVICE = -5     /* a HIP call failed */
} hh_status;

typedef enum { HH_F32 = 0, HH_BF16 = 1 } hh_dtype;

/* hh_cfg.kernel_flags: each bit routes a family of launches to the slower kernel that computes the
 * same thing, so that tests can compare the two (results agree to float32 rounding order). */
enum {
  HH_KF_ATTN_SCALAR = 1,   /* bf16 cache: attention on the vector ALU instead of the matrix cores */
  HH_KF_SSM_GENERAL = 2,   /* the any-length scan kernel also for passes of at most 9 positions */
  HH_KF_MID_OFF = 4,       /* 17..96 activation rows through the many-row GEMM */
  HH_KF_SKINNY_OFF = 8,    /* 4..16 activation rows through the FMA kernel (4..8) and the many-row GEMM (9..16) */
  HH_KF_SSM_SCALAR_CONV = 16, /* prefill scan: element-wise staging of the convolution inputs */
  HH_KF_ROWS_LDS = 32,     /* with HH_KF_MID_OFF: 17..96 activation rows through the LDS-staged many-row GEMM */
  HH_KF_SSM_SEQUENTIAL = 64, /* passes of 16 and more positions: the position-by-position scan instead of the matmul form */
  HH_KF_NO_HANDOVER = 128, /* many-row passes: the SwiGLU result goes through float32 and a split kernel to the down projection */
  HH_KF_SSM_MATMUL = 512,  /* the matmul form of the scan also for launches of fewer than 128 workgroups (default: the sequential kernel there) */
  HH_KF_MID_WIDE = 1024,   /* 17..80 activation rows: the 8-wavefront, 128-column-window shape of the 81..96-row products (one workgroup per compute unit) */
  HH_KF_CANARIES = 256     /* every region the library carves from the workspace is followed by 256 guard bytes (see hh_check_canaries) */
};

/* Model shape and capacities.  Plain data; set struct_size = sizeof(hh_cfg). */
typedef struct hh_cfg {
  uint32_t struct_size;
  int32_t n_layers, d_model, vocab;
  int32_t m_heads, m_head_dim, d_state; /* Mamba-2 branch: heads x head_dim = d_inner, state size N */
  int32_t n_groups;                     /* must be 1 */
  int32_t d_conv;                       /* causal depthwise conv taps, must be 4 */
  int32_t n_q_heads, n_kv_heads, head_dim; /* attention branch; n_q_heads % n_kv_heads == 0, head_dim even */
  float rope_base;
  int32_t d_ff;                         /* SwiGLU width */
  float rms_eps;
  int32_t w_dtype;                      /* hh_dtype of matrices and of the KV cache */
  int32_t max_batch;                    /* sequences per prefill */
  int32_t max_seq_len;                  /* per sequence: prompt + max_new + 2*max_draft + 2 must fit */
  int32_t max_draft;                    /* largest k */
  int32_t max_new_tokens;               /* largest generation budget per sequence */
  int32_t kv_page_tokens;               /* tokens per KV page: 16, 32, 64, 128 or 256; 0 = default */
  int32_t prefill_chunk;                /* prompt positions per sequence per prefill pass, 1..1024; 0 = default:
                                           4096 / max_batch rounded down to a multiple of 64, within 64..512 */
  int32_t keep_logits;                  /* 1: float32 logits of the draft, verification and last prefill rows are kept for
                                           hh_get_logits.  0: greedy rounds (temperature 0) keep only the argmax of every
                                           row - the LM head of a pass with more than 16 rows then writes no logits at
                                           all - and hh_get_logits returns HH_ESTATE; at temperature > 0 the rows are
                                           written regardless (Eq. 6 reads them) */
  int32_t use_graphs;                   /* 1: the launch sequences of hh_draft and hh_verify are replayed as HIP graphs from
                                           their second use on (non-NULL stream only); hh_commit is always enqueued directly */
  /* Tunables: results must not depend on them beyond float32 rounding order (0 = the library's default). */
  int32_t overlap_mode;                 /* attention branch of a full pass on a side stream beside the SSM branch:
                                           0 automatic (= 2), 1 never, 2 prefill passes only, 3 always */
  int32_t attn_max_splits;              /* most key slices (workgroups along the cache) per sequence and KV head: 1..32; 0 = 16 */
  int32_t attn_target_blocks;           /* key slices are chosen so that an attention launch has about this many workgroups
                                           (sequences x KV heads x row chunks x slices): 64..8192; 0 = 256 */
  int32_t attn_single_slice_steps;      /* matrix-core attention: caches of at most this many 32-key steps use one slice;
                                           0 = 28, -1 = split from the first step on */
  int32_t kernel_flags;                 /* HH_KF_* bits: kernel selection for cross-checks, all 0 by default */
  int32_t prefill_progress;             /* n > 0: hh_prefill waits for every n-th pass and reports it on stderr */
  int32_t draft_state_mode;             /* recurrent state the draft model M_S runs on (Eq. 4, Section 3.3 draft phase):
                                           0 shared: every round's draft starts from the full model's committed state;
                                           1 strict: M_S is a model of its own over the whole prefix - a second committed
                                             state and ring per layer, advanced with attention suppressed over the prompt
                                             (one more SSM-only pass per prefill chunk) and over every committed token
                                             (hh_draft runs k+1 SSM-only steps, the last without LM head; hh_commit
                                             rebuilds both states).  The committed stream is the same; accepted counts differ */
  void* workspace;                      /* DEVICE, 256-byte aligned */
  size_t workspace_bytes;
} hh_cfg;

/* DEVICE pointers to one block's weights (Eq. 2: both branches read the same
 * normalised input; the block also carries its SwiGLU MLP). */
typedef struct hh_layer_weights {
  const void* norm1;   /* f32 [d_model]               shared input RMSNorm */
  const void* w_in;    /* w   [d_in_proj][d_model]    rows: z(d_inner) | x(d_inner) B(N) C(N) | dt(m_heads) */
  const void* conv_w;  /* f32 [conv_dim][d_conv]      tap j multiplies the input d_conv-1-j positions back */
  const void* conv_b;  /* f32 [conv_dim] */
  const void* a_log;   /* f32 [m_heads]               A = -exp(a_log) */
  const void* d_skip;  /* f32 [m_heads] */
  const void* dt_bias; /* f32 [m_heads] */
  const void* gnorm;   /* f32 [d_inner]               RMSNorm applied to y * silu(z) */
  const void* w_out;   /* w   [d_model][d_inner] */
  const void* w_q;     /* w   [n_q_heads*head_dim][d_model] */
  const void* w_k;     /* w   [n_kv_heads*head_dim][d_model] */
  const void* w_v;     /* w   [n_kv_heads*head_dim][d_model] */
  const void* w_o;     /* w   [d_model][n_q_heads*head_dim] */
  const void* norm2;   /* f32 [d_model] */
  const void* w_gate;  /* w   [d_ff][d_model] */
  const void* w_up;    /* w   [d_ff][d_model] */
  const void* w_down;  /* w   [d_model][d_ff] */
} hh_layer_weights;

typedef struct hh_weights {
  const void* embed;      /* w   [vocab][d_model]   DEVICE */
  const void* final_norm; /* f32 [d_model]          DEVICE */
  const void* lm_head;    /* w   [vocab][d_model]   DEVICE */
  const hh_layer_weights* layers; /* HOST array of n_layers entries (copied by hh_create) */
} hh_weights;

/* Bytes of device workspace needed for cfg (workspace fields ignored); 0 if cfg is invalid. */
HH_API size_t hh_workspace_bytes(const hh_cfg* cfg);

/* Validates cfg, carves the workspace, builds the RoPE table and, for bf16 weights, the library's
 * own copies of the matrices (stacked input projections; every matrix repacked into matrix-core
 * operand tiles): the workspace therefore holds about 1.2x the matrix bytes besides the caches.
 * The caller's weights must stay valid and unchanged while the context lives.  *out is NULL on failure. */
HH_API hh_status hh_create(const hh_weights* weights, const hh_cfg* cfg, hh_ctx** out);
HH_API hh_status hh_destroy(hh_ctx* ctx);

/* Run M_H over the prompts (Section 3.3: the prefix x_{1:t}), fill the KV cache
 * and the recurrent state, and take the first generated token as each
 * sequence's pending token (emitted, not yet consumed by the caches).
 *   tokens      DEVICE int32 [batch][row_stride], ids in [0, vocab) (the library cannot check device
 *               data: an id outside the range is read as the nearest valid one)
 *   lens        HOST   int32 [batch], 1 <= lens[b] <= row_stride
 *   max_new     generation budget per sequence (1 .. cfg.max_new_tokens)
 * Resets every sequence slot.  HH_ECAPACITY if lens[b] + max_new + 2*max_draft + 2
 * exceeds max_seq_len or batch exceeds max_batch. */
HH_API hh_status hh_prefill(hh_ctx* ctx, const int32_t* tokens, int32_t row_stride, const int32_t* lens,
                     int32_t batch, int32_t max_new, void* stream);

/* Temperature of the token choice (Section 3.3, Eq. 6; the paper evaluates T = 0 and T = 0.6).
 * temperature = 0 (the state after hh_create): greedy, every call as described at that call.
 * temperature > 0: P = softmax(logits / temperature); the first token and every draft token are
 * drawn from their distribution, hh_verify applies the rejection test of Eq. 6 to the drafts
 * in order (draft d kept with probability min(1, P_H(d) / P_S(d))), and the token emitted after
 * the n kept drafts is drawn from norm(max(0, P_H - P_S)) at the first rejection, or from P_H at
 * position k+1 when all are kept.  hh_verify then leaves, in place of M_H's argmaxes, targets
 * g_i = d_{i+1} for i < n, g_n = the emitted token and -1 behind it, so that hh_commit's prefix
 * rule returns n.  A draw from p with a uniform u takes the smallest index i with
 * p_0 + .. + p_i > u * sum(p).  Uniforms: the top 24 bits of output number c of SplitMix64
 * started at `seed`, c = sequence * 2^34 + position in the generated stream * 4 + purpose
 * (0 draft draw, 1 acceptance test, 2 emitted / first token): HOST scalars, nothing kept from the
 * caller.  At temperature > 0 hh_set_drafts and a forced count in hh_commit return HH_ESTATE.
 * Valid before hh_prefill and between rounds (HH_ESTATE inside a round); synchronises `stream`.
 * HH_EINVAL for a negative or non-finite temperature. */
HH_API hh_status hh_set_sampling(hh_ctx* ctx, float temperature, uint64_t seed, void* stream);

/* The two steps of the temperature > 0 token choice on caller-provided logits, without a
 * context (the same kernels hh_draft and hh_verify launch after hh_set_sampling; Eq. 6).  All
 * pointers DEVICE, float32 logits, nothing is kept.  HH_EINVAL for NULL or out-of-range
 * arguments or a temperature that is not finite and > 0; HH_EDEVICE if a launch fails.
 *
 * hh_draw_tokens: out[r] = a draw from softmax(logits[r * row_stride ..][0..vocab) / temperature)
 * with the uniform of (seed, sequence r, position (positions ? positions[r] : 0) + position_offset,
 * purpose): the smallest index whose cumulative mass exceeds u times the total.
 *
 * hh_accept_tokens: for every sequence b, the rejection test over drafts[b][0..k) with
 * draft_logits [batch][k][vocab] and verify_logits [batch][k+1][vocab] and the token emitted after
 * the n kept drafts; positions[b] is the stream position of the first draft (uniforms: purpose 1 at
 * positions[b] + i for test i, purpose 2 at positions[b] + n for the emitted token).  Writes
 * targets [batch][k+1]: drafts[b][i] for i < n, the emitted token at n, -1 behind it.  A draft id
 * outside [0, vocab) counts as rejected.
 * scratch: batch * (2k+1) * 2 floats. */
HH_API hh_status hh_draw_tokens(const float* logits, int64_t row_stride, int32_t vocab, int32_t rows, float temperature,
                                uint64_t seed, const int32_t* positions, int32_t position_offset, int32_t purpose,
                                int32_t* out, void* stream);
HH_API hh_status hh_accept_tokens(const float* draft_logits, const float* verify_logits, int32_t vocab, int32_t batch,
                                  int32_t k, const int32_t* drafts, const int32_t* positions, float temperature,
                                  uint64_t seed, float* scratch, int32_t* targets, void* stream);

/* hh_accept_tokens for callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without
 * `scratch`, same kernels, same result.  The per-row softmax statistics live in an array built
 * into the library (256 KiB of device memory per GPU, held until the process ends); the call
 * allocates nothing.  HH_ECAPACITY if batch * (2k + 1) * 2 exceeds 65536 floats (e.g. 64 sequences
 * with k = 8 need 2176); the message is available from hh_last_error(NULL).  Every entry the
 * kernels read is written first, so nothing has to be cleared between calls; calls that overlap on
 * one GPU (different streams or threads) share the array and race - serialise them. */
HH_API hh_status hh_accept_tokens_static(const float* draft_logits, const float* verify_logits, int32_t vocab, int32_t batch,
                                         int32_t k, const int32_t* drafts, const int32_t* positions, float temperature,
                                         uint64_t seed, int32_t* targets, void* stream);

/* Draft phase (Section 3.3 / Eq. 4): k autoregressive greedy steps of the
 * SSM-only subgraph per sequence, starting from the committed recurrent state
 * on a scratch copy; never touches the KV cache.  0 <= k <= max_draft; k = 0
 * makes the round a plain greedy step of M_H.  With draft_state_mode = 1 the
 * steps start from M_S's own committed state and one more step (no LM head)
 * consumes d_k; with a draft mask (hh_set_draft_mask) layers marked
 * HH_DRAFT_FULL also run their attention branch and write K/V into the slots
 * behind the cache length, layers marked HH_DRAFT_SKIP are passed over. */
HH_API hh_status hh_draft(hh_ctx* ctx, int32_t k, void* stream);

/* Replace the drafted tokens of the current round by caller-chosen ones
 * (DEVICE int32 [batch][k]); valid between hh_draft and hh_verify.  The
 * committed stream does not depend on the draft source (losslessness).
 * With draft_state_mode = 1 the call also runs M_S (no LM head) over the
 * replaced tokens, so that its state follows what is committed. */
HH_API hh_status hh_set_drafts(hh_ctx* ctx, const int32_t* drafts, void* stream);

/* Draft model by layers (Section 4.2: layer-skipping and early-exit drafts; Eq. 5 applied to whole
 * blocks).  modes: HOST int32 [n_layers], one of
 *   HH_DRAFT_SSM   only the SSM branch of the block runs (Eq. 4; the default for every layer),
 *   HH_DRAFT_FULL  both branches run as in M_H: the draft step attends over the cache and writes its
 *                  K/V at the position it drafts (a slot behind the cache length, rewritten by hh_verify),
 *   HH_DRAFT_SKIP  the block is the identity on the residual stream; its state is not touched.
 * NULL restores the default.  Copied; applies to the following hh_draft calls.  The committed stream
 * never depends on the mask.  HH_ESTATE inside a round, or for a mask other than all-SSM on a context
 * with draft_state_mode = 1; HH_EINVAL for an unknown mode. */
enum { HH_DRAFT_SSM = 0, HH_DRAFT_FULL = 1, HH_DRAFT_SKIP = 2 };
HH_API hh_status hh_set_draft_mask(hh_ctx* ctx, const int32_t* modes);

/* The draft length among candidates[0..n_candidates) (HOST, each >= 0) that maximises the speedup
 * model of Eq. 1, (1 - alpha^(k+1)) / ((1 - alpha) (1 + k * cost_ratio)), for per-token acceptance
 * probability alpha in [0, 1] and cost_ratio = c_draft / c_verify >= 0 (Section 7, optimal draft
 * length); the shortest of equally good lengths.  Host arithmetic only.  -1 for bad arguments. */
HH_API int32_t hh_optimal_draft_length(double alpha, double cost_ratio, const int32_t* candidates, int32_t n_candidates);

/* Verification phase (Section 3.3): one pass of M_H over pending, d_1..d_k at
 * positions len..len+k of every sequence: chunked SSM scan from the committed
 * state with the data needed to restore the state after any position, K/V
 * appended to the paged cache, causal attention over len+j+1 keys, and M_H's
 * argmax g_j for j = 0..k. */
HH_API hh_status hh_verify(hh_ctx* ctx, void* stream);

/* Greedy acceptance and rollback (Section 3.3): n = longest prefix with
 * d_i == g_{i-1}; emit d_1..d_n, g_n (clamped to the budget); pending = g_n;
 * recurrent state = state after position n; cache length += n+1 (later slots
 * are dead).  n_accepted: NULL for the greedy rule, else DEVICE int32 [batch]
 * with 0 <= n <= k taken as given (drafts committed as drafted).  Sequences
 * that have reached their budget are left untouched. */
HH_API hh_status hh_commit(hh_ctx* ctx, const int32_t* n_accepted, void* stream);

/* ---- read-back (HOST output pointers; synchronise `stream`) ---- */
/* Committed tokens of sequence seq (first generated token first). */
HH_API hh_status hh_get_tokens(hh_ctx* ctx, int32_t seq, int32_t* out, int32_t cap, int32_t* n_out, void* stream);
/* Per sequence: cache length, committed count, accepted count of the last commit.  Any pointer may be NULL. */
HH_API hh_status hh_get_lengths(hh_ctx* ctx, int32_t* kv_len, int32_t* committed, int32_t* last_n, void* stream);
/* Contexts created with HH_KF_CANARIES: checks the guard bytes behind every region of the workspace
 * (a kernel that writes past the end of its buffer damages them).  *n_damaged (HOST) = number of
 * damaged guards; hh_last_error names the first.  Synchronises `stream`.  HH_ESTATE without the flag. */
HH_API hh_status hh_check_canaries(hh_ctx* ctx, int32_t* n_damaged, void* stream);
/* Acceptance statistics since the last hh_prefill, summed over rounds and unfinished sequences:
 * *accepted = drafts that passed their test (sum of n), *tested = drafts that were tested (in a round
 * with k drafts and n accepted: min(n + 1, k) - the first rejected draft is the last one tested).
 * accepted / tested is the maximum-likelihood estimate of the per-token acceptance probability alpha
 * of Eq. 1, the input of hh_optimal_draft_length for choosing k round by round (Section 7: adaptive
 * draft length).  Forced counts are counted as given. */
HH_API hh_status hh_get_acceptance(hh_ctx* ctx, uint64_t* accepted, uint64_t* tested, void* stream);
/* Tokens of the current round: drafts [batch][k] and targets g [batch][k+1] (M_H's argmaxes; at
 * temperature > 0 the kept drafts, the emitted token and -1 behind it).  Either may be NULL. */
HH_API hh_status hh_get_round(hh_ctx* ctx, int32_t* drafts, int32_t* targets, void* stream);
/* Logits (needs cfg.keep_logits): which = 0 draft rows [batch][k][vocab], 1 verify rows
 * [batch][k+1][vocab], 2 prefill last-position rows [batch][vocab]. */
HH_API hh_status hh_get_logits(hh_ctx* ctx, int32_t which, float* out, void* stream);
/* Committed recurrent state of one layer: ssm [batch][m_heads][m_head_dim][d_state],
 * conv [batch][conv_dim][d_conv-1] (oldest first).  Either may be NULL. */
HH_API hh_status hh_get_state(hh_ctx* ctx, int32_t layer, float* ssm, float* conv, void* stream);
/* The same for the draft model's own committed state (draft_state_mode = 1; HH_ESTATE otherwise). */
HH_API hh_status hh_get_draft_state(hh_ctx* ctx, int32_t layer, float* ssm, float* conv, void* stream);
/* First n_tokens cache entries of one sequence and layer as float32 [n_tokens][n_kv_heads][head_dim]. */
HH_API hh_status hh_get_kv(hh_ctx* ctx, int32_t layer, int32_t seq, int32_t n_tokens, float* k, float* v, void* stream);

/* ---- optional per-launch timing (for measurement; perturbs throughput, keep it out of timed runs) ----
 * While enabled, every kernel launch of prefill/draft/verify/commit is bracketed by a HIP event
 * pair on the call's stream, tagged  phase * 16 + kind.  Enabling clears earlier records. */
enum { HH_PHASE_PREFILL = 0, HH_PHASE_DRAFT = 1, HH_PHASE_VERIFY = 2, HH_PHASE_COMMIT = 3 };
enum { HH_K_IN_PROJ = 0, HH_K_SSM = 1, HH_K_RESERVED = 2, HH_K_ATTN = 3, HH_K_OUT_PROJ = 4, HH_K_O_PROJ = 5,
       HH_K_MLP_UP = 6, HH_K_MLP_DOWN = 7, HH_K_LM_HEAD = 8 };
HH_API hh_status hh_profile(hh_ctx* ctx, int32_t enable);
/* Synchronises `stream`; launches[tag] and total_ms[tag] (HOST, n_tags entries, tag as above)
 * receive the number of timed launches and their summed duration. */
HH_API hh_status hh_profile_read(hh_ctx* ctx, int32_t n_tags, int32_t* launches, float* total_ms, void* stream);

/* Launch duration of one kind of kernel in its place: enqueues `reps` draft (phase HH_PHASE_DRAFT)
 * or verification (HH_PHASE_VERIFY, k+1 positions) passes in which ONLY kernels of `kind` are
 * launched (so consecutive launches read different layers' weights, as in a real pass), between
 * one HIP event pair on `stream`; synchronises.  *total_ms / *launches is the average duration
 * including the launch gap.  Valid between rounds; activations and draft scratch are left
 * undefined, committed state is untouched.  HOST outputs. */
HH_API hh_status hh_time_kind(hh_ctx* ctx, int32_t phase, int32_t kind, int32_t k, int32_t reps, float* total_ms,
                              int32_t* launches, void* stream);

/* Human-readable description of the last error on this context (or, when ctx is NULL, of the
 * last failed context-free call: hh_create, hh_workspace_bytes, ...).  Never NULL. */
HH_API const char* hh_last_error(const hh_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* HH_H */
