/*
 * fly.h -- C ABI of the FLy verification step on one MI355X (gfx950).
 *
 * FLy (Training-Free Loosely Speculative Decoding, arxiv 2511.22972) changes
 * only how the target model verifies a block of K draft tokens.  This library
 * is that verification step: one forward pass of a Llama-style decoder over
 * the K+1 tokens (y_{-1}, draft_1..draft_K) against a cached prefix (paper
 * Sec. 2.1; Algorithm 1 step 2), per-position softmax statistics (Eq. 1,
 * Eq. 5), and the loose acceptance rule (Eqs. 2-11; Algorithm 1 steps 3-4).
 *
 * General conventions
 *   - Every function returns a fly_status (0 = OK, negative = error) and never
 *     throws, aborts, allocates or synchronises.  All GPU work is enqueued on
 *     the caller's stream (`fly_stream` is a hipStream_t; NULL = default
 *     stream).
 *   - Pointers marked [device] are device memory owned by the caller and must
 *     stay valid until the enqueued work has finished; they must be 16-byte
 *     aligned.  Pointers marked [host] are read during the call only.
 *   - Arguments are validated on the host before anything is enqueued; on an
 *     error nothing has been launched.
 *   - M = B*(K+1) rows; row m = b*(K+1) + i is position i of sequence b and
 *     sits at absolute position kv_len[b] + i.  1 <= B <= 65536 and 1 <= K <= 63
 *     (FLY_ERR_BAD_SHAPE / FLY_ERR_K_RANGE otherwise).
 *   - dtype FLY_F32: weights, KV cache and activations are fp32.
 *     dtype FLY_BF16: weights, KV cache and GEMM operands are bf16, the
 *     residual stream, accumulators and all statistics are fp32.
 */
#ifndef FLY_H
#define FLY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FLY_OK = 0,
  FLY_ERR_NULL_POINTER = -1,   /* a required pointer is NULL */
  FLY_ERR_BAD_SHAPE = -2,      /* B, M, d, F, V, heads ... out of range or not tileable */
  FLY_ERR_K_RANGE = -3,        /* K outside [1, 63] (one wavefront holds a block) */
  FLY_ERR_WINDOW = -4,         /* W < 0 */
  FLY_ERR_THETA = -5,          /* theta is NaN */
  FLY_ERR_DTYPE = -6,          /* unknown fly_dtype */
  FLY_ERR_HEAD_DIM = -7,       /* head_dim not supported for this dtype */
  FLY_ERR_ALIGNMENT = -8,      /* a device pointer is not 16-byte aligned */
  FLY_ERR_WORKSPACE = -9,      /* workspace NULL or smaller than the query says */
  FLY_ERR_KV_CAPACITY = -10,   /* max_kv_len + K + 1 exceeds the cache capacity */
  FLY_ERR_LAUNCH = -11,        /* the HIP runtime refused a launch */
  FLY_ERR_STATIC_SCRATCH = -12 /* the request does not fit the library's static scratch array */
} fly_status;

typedef enum { FLY_F32 = 0, FLY_BF16 = 1 } fly_dtype;

typedef void* fly_stream; /* hipStream_t */

/* Geometry of the target model (shapes only; the paper fixes none of them). */
typedef struct {
  int32_t n_layers;
  int32_t d;          /* hidden size */
  int32_t n_q_heads;  /* Hq */
  int32_t n_kv_heads; /* Hkv, divides Hq */
  int32_t head_dim;   /* hd: 64 or 128 for FLY_F32, 128 for FLY_BF16 */
  int32_t ffn;        /* F, SwiGLU width */
  int32_t vocab;      /* V = |vocabulary| of Eq. 5 */
  int32_t dtype;      /* fly_dtype */
  float rms_eps;
  float rope_theta;
} fly_model_desc;

/*
 * Packed weights of one decoder layer [device].  Each matrix was produced by
 * fly_pack_weight from a canonical row-major [in, out] matrix:
 *   w_qkv     [d, (Hq+2Hkv)*hd]  columns = q heads, then k heads, then v heads
 *   w_o       [Hq*hd, d]
 *   w_gateup  [d, 2F]            16-column tiles alternate gate, up, gate, up ...
 *   w_down    [F, d]
 *   g_attn, g_ffn  RMSNorm gains [d] in the model dtype
 */
typedef struct {
  const void* w_qkv;
  const void* w_o;
  const void* w_gateup;
  const void* w_down;
  const void* g_attn;
  const void* g_ffn;
} fly_layer_weights;

typedef struct {
  const void* embed;                /* [device] [V, d] row-major, model dtype */
  const fly_layer_weights* layers;  /* [host] array of n_layers entries */
  const void* g_final;              /* [device] final RMSNorm gain [d] */
  const void* w_lm;                 /* [device] packed [d, V] */
} fly_weights;

/*
 * KV cache.  Per layer, keys are [B, Hkv, capacity, hd] and values are stored
 * transposed, [B, Hkv, hd, capacity], both in the model dtype; keys are held
 * already rotated.  Rows 0..kv_len[b]-1 of sequence b are the cached prefix.
 * The verification step writes rows kv_len[b]..kv_len[b]+K of every layer and
 * reads rows 0..kv_len[b]+K.  capacity must be a multiple of 64.
 */
typedef struct {
  void* const* k_layers;   /* [host] n_layers device pointers */
  void* const* v_layers;   /* [host] n_layers device pointers */
  const int32_t* kv_len;   /* [device] int32 [B] */
  int32_t capacity;        /* rows allocated per sequence */
  int32_t max_kv_len;      /* host-side bound: kv_len[b] <= max_kv_len for all b */
} fly_kv_cache;

/* Outputs of fly_verify_block, all [device]; the last three may be NULL. */
typedef struct {
  int32_t* accept_len;   /* [B]  draft tokens kept = s_FLy - 1  (Eq. 11) */
  int32_t* next_token;   /* [B]  y_s: correction token, or the bonus token when all K are kept */
  int32_t* kv_len_out;   /* [B]  kv_len + accept_len + 1 (rows of the cache that stay valid) */
  int32_t* argmax;       /* [B, K+1] target tokens y_1..y_{K+1} (Eq. 1) */
  float* h_norm;         /* [B, K+1] normalised entropy (Eq. 5) */
  float* p_top1;         /* [B, K+1] probability of the argmax token */
  float* lse;            /* [B, K+1] log-sum-exp of the row, nullable */
  int32_t* n_loose;      /* [B] mismatching drafts that were kept, nullable */
  float* hidden_out;     /* [M, d] fp32 residual stream after the last layer, nullable */
} fly_verify_out;

const char* fly_strerror(fly_status s);

/*
 * Launch-shape knobs for experiments (process-wide; a change made while another thread plans a
 * call is seen by that call or by the next):
 *   "gemm_nt"      16-column weight tiles per wavefront: 1, 2, 4; 0 = automatic
 *   "gemm_splits"  split-K factor of the projections: 1..16; 0 = automatic
 *   "gemm_mt_max"  most 16-row activation tiles one workgroup holds: 5 or 9 (default 9)
 *   "gemm_tiled"   0 = the LDS-tiled GEMM above 256 rows (automatic), 1 = never,
 *                  2, 3, 4 or 6 = always, with workgroups of 128, 192, 256 or 384 rows
 *   "gemm_wide"    0 = the weight-streaming GEMM with 32-row tiles for 81..256 rows (automatic),
 *                  1 = never, 3, 4, 5, 6 or 8 = always, with that many 32-row tiles (M must fit)
 *   "wide_phase"   the same GEMM: 1 = half of the waves request their loads after multiplying,
 *                  2 = every wave before; 0 = automatic (1 from four row tiles on)
 *   "tiled_phase"  the LDS-tiled GEMM: 1 = the odd waves request their loads between the two halves
 *                  of a step's multiplies, 2 = every wave first; 0 = automatic (1)
 *   "attn_splits"  cache splits per (sequence, KV head): 1..256; 0 = automatic
 *   "attn_block_tiles"  most 32-row query tiles per workgroup: 1..8; 0 = automatic (8)
 *   "attn_phase"   1 = the odd waves request their share of the next cache stage after multiplying,
 *                  2 = every wave first; 0 = automatic (1)
 *   "target_wgs"   workgroups a launch aims for (default 256, one per compute unit)
 * Workspace sizes depend on them: query again after a change.
 */
fly_status fly_set_tuning(const char* key, int32_t value);

/*
 * Weight packing (one-time, at load).  The packed layout is this library's own:
 *   FLY_BF16: tiles of 16 output columns x 32 input rows, each stored as the 64
 *             lanes x 8 values one matrix-core operand load wants, tiles of
 *             one 16-column strip contiguous along the input dimension.
 *             Requires k_in % 32 == 0.
 *   FLY_F32:  row-major [k_in, n_dst].
 * Source column tile j (columns 16j..16j+15 of src [k_in, n_src] row-major)
 * lands at destination column tile tile_offset + j*tile_stride of a
 * destination that is n_dst columns wide.  n_src and n_dst must be multiples
 * of 16.  fly_packed_weight_bytes gives the destination size.
 */
fly_status fly_packed_weight_bytes(int64_t k_in, int64_t n_dst, int32_t dtype, size_t* bytes);
fly_status fly_pack_weight(const void* src /*[device]*/, int64_t k_in, int64_t n_src, int32_t dtype,
                           void* dst /*[device]*/, int64_t n_dst, int64_t tile_offset,
                           int64_t tile_stride, fly_stream stream);

/* Workspace sizes (bytes) for the calls below. */
fly_status fly_workspace_bytes(const fly_model_desc* desc, int32_t B, int32_t K,
                               int32_t max_kv_len, size_t* bytes);
fly_status fly_lmhead_workspace_bytes(int32_t M, int32_t d, int32_t V, int32_t dtype, size_t* bytes);

/*
 * The verification step (paper Sec. 2.1-2.2; Algorithm 1 steps 2-4).
 *   tokens     [device] int32 [B, K+1] = y_{-1}, draft_1..draft_K per sequence
 *   row_scale  [device] float [B*(K+1)] multiplier applied to each row's logits
 *              before the statistics (1/temperature of the synthetic
 *              workloads), or NULL for 1
 *   theta, W   entropy threshold and deferred-window length of Eqs. 6-9
 * Runs embedding, n_layers decoder layers (appending K+1 rows per layer to the
 * KV cache), the final norm, the LM head with fused row statistics -- the
 * logits are never written to memory -- and the acceptance rule.
 * Errors: see fly_status; K > 63 is FLY_ERR_K_RANGE.
 */
fly_status fly_verify_block(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                            const int32_t* tokens, const float* row_scale, int32_t B, int32_t K,
                            float theta, int32_t W, const fly_verify_out* out, void* workspace,
                            size_t workspace_bytes, fly_stream stream);

/*
 * The verification step at temperature > 0.  The paper reports temperature-1
 * results (Tables 1-2) and states its rule with the argmax only (Eqs. 1-2);
 * this entry point takes the reading that the target's token y_i is DRAWN from
 * softmax(row_scale[m] * logits[m]) and takes the argmax's place in the match
 * indicator of Eq. 2, while the entropy gate (Eqs. 5-6) reads the same tempered
 * distribution.  Everything else is fly_verify_block.
 *   seed, offset  the draw of row m = b*(K+1) + i and column v is the Gumbel-max
 *                 construction, argmax_v (logit_v + G_v), G_v = -ln(-ln u_v), with
 *                 u_v = (top 23 bits + 1/2) / 2^23 of word v % 4 of the
 *                 Philox4x32-10 block with counter (v / 4, m, offset low word,
 *                 offset high word) and key (seed low word, seed high word).  Give
 *                 every call of a run its own offset (a round counter, say).
 *   sampled       [device] int32 [B, K+1]: the drawn tokens y_1..y_{K+1}; the
 *                 acceptance rule compares the drafts with these, next_token is
 *                 one of them.  out->argmax still receives the argmax.
 * The logits are still never written to memory: the draw is one more statistic
 * fused into the LM head.  Same workspace as fly_verify_block.
 */
fly_status fly_verify_block_sampled(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                                    const int32_t* tokens, const float* row_scale, int32_t B, int32_t K,
                                    float theta, int32_t W, uint64_t seed, uint64_t offset,
                                    int32_t* sampled, const fly_verify_out* out, void* workspace,
                                    size_t workspace_bytes, fly_stream stream);

/*
 * The sequences of a multi-round decode (Algorithm 1: y, and the counters s, t).
 * Row b of ctx holds y of sequence b: the prompt followed by everything emitted
 * so far; ctx_len[b] tokens are valid.  The last token of a row is y_{-1}: it
 * is not yet in the KV cache, so kv_len[b] == ctx_len[b] - 1 must hold on entry
 * (the cache of a synthetic prefix may of course not be the cache of these
 * tokens; only the lengths must agree).  All arrays [device]; statistics may
 * be NULL and are ACCUMULATED (zero them before the first call).
 */
typedef struct {
  int32_t* ctx;             /* [B, ctx_capacity] int32 */
  int32_t* ctx_len;         /* [B] advanced by s every round */
  int32_t* kv_len;          /* [B] the cache lengths; must be the array the fly_kv_cache points to */
  int32_t ctx_capacity;     /* tokens per row */
  int32_t max_ctx_len;      /* host-side bound: ctx_len[b] <= max_ctx_len on entry */
  int64_t* accepted_total;  /* [B] sum of s over the rounds (Algorithm 1's s), nullable */
  int32_t* rounds_done;     /* [B] Algorithm 1's t, nullable; tau = accepted_total / rounds_done (Eq. 12) */
  int64_t* loose_total;     /* [B] mismatching drafts that were kept, nullable */
  int32_t* accept_trace;    /* [rounds, B] s of every round of this call, nullable */
  int32_t* ngram_trace;     /* [rounds, B] n-gram length the drafter matched (0: none), nullable */
} fly_sequences;

/*
 * Prompt-lookup drafting (Sec. 2.3 names n-gram retrieval over the context as
 * the parameter-free drafter; the rule is this library's).  For every sequence:
 * the longest n <= ngram_max such that the last n tokens occur earlier in the
 * sequence wins, among its occurrences the latest; the K tokens following it
 * are proposed, continuing through the proposal itself where the copy runs past
 * the end; without any occurrence the last token is repeated.
 *   ctx [device] int32 [B, ctx_capacity], ctx_len [device] int32 [B], 1 <= ctx_len[b] <= ctx_capacity
 *   tokens [device] int32 [B, K+1]: (last token, draft_1..draft_K), the block fly_verify_block takes
 *   ngram  [device] int32 [B], nullable: the n that matched (0: none)
 * 1 <= K <= 63, 1 <= ngram_max <= 64.  Integer-only, deterministic.
 */
fly_status fly_pld_draft(const int32_t* ctx, const int32_t* ctx_len, int32_t ctx_capacity, int32_t B,
                         int32_t K, int32_t ngram_max, int32_t* tokens, int32_t* ngram,
                         fly_stream stream);

/*
 * `rounds` rounds of Algorithm 1 on the device, without a host round trip:
 * draft K tokens by prompt lookup (fly_pld_draft), verify them
 * (fly_verify_block: forward, row statistics, loose acceptance), then append
 * the kept drafts and the correction / bonus token to the sequences and move
 * the cache lengths to the rows that stay valid (kv_len += s).  There is no
 * end-of-sequence token in this setting: the loop runs the given number of
 * rounds.  row_scale (nullable) is applied to the K+1 rows of every round.
 * The host-side bounds must leave room for the whole call:
 *   kv->max_kv_len + rounds*(K+1) <= kv->capacity,
 *   seq->max_ctx_len + rounds*(K+1) <= seq->ctx_capacity,
 * else FLY_ERR_KV_CAPACITY.  kv->kv_len must be seq->kv_len (it is written).
 * Workspace: fly_decode_workspace_bytes(desc, B, K, kv->max_kv_len + rounds*(K+1)).
 */
fly_status fly_decode_workspace_bytes(const fly_model_desc* desc, int32_t B, int32_t K,
                                      int32_t max_kv_len_end, size_t* bytes);
fly_status fly_decode_rounds(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                             const fly_sequences* seq, const float* row_scale, int32_t B, int32_t K,
                             float theta, int32_t W, int32_t ngram_max, int32_t rounds,
                             void* workspace, size_t workspace_bytes, fly_stream stream);

/*
 * The same loop at temperature > 0: every round is fly_verify_block_sampled
 * (which see, also for what this reading of the paper is), round r of the call
 * drawing with offset + r; give consecutive calls of one run offsets `rounds`
 * apart.  The drafter is unchanged.  Same workspace.
 */
fly_status fly_decode_rounds_sampled(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                                     const fly_sequences* seq, const float* row_scale, int32_t B, int32_t K,
                                     float theta, int32_t W, int32_t ngram_max, int32_t rounds,
                                     uint64_t seed, uint64_t offset, void* workspace,
                                     size_t workspace_bytes, fly_stream stream);

/*
 * Drafting with a draft model M_D (Algorithm 1 step 1 in the paper's own setting:
 * a small model of the target's family proposes, the target verifies).  For every
 * sequence b with n = ctx_len[b] tokens: the K tokens M_D emits greedily after
 * them (Eq. 1 with M_D's distribution, lowest index on ties), by K forward passes
 * of M_D that chain on the device.
 *   desc, w, kv   the draft model, its packed weights and its OWN cache.  Only the
 *                 layer pointers and the capacity of kv are used: the rows before
 *                 position n-2 must be M_D's rows of the sequence so far (or a
 *                 synthetic prefix); the rows of the last two tokens are computed
 *                 (again) by every call, then the rows of draft_1..draft_{K-1}.
 *                 So the cache needs no roll-back after a rejection: whatever the
 *                 target kept, the next call finds valid rows before its n-2.
 *   ctx, ctx_len  [device] as in fly_sequences; 2 <= ctx_len[b] <= max_ctx_len (host bound)
 *   tokens        [device] int32 [B, K+1]: (last token, draft_1..draft_K)
 * kv->capacity must be at least max_ctx_len + K, else FLY_ERR_KV_CAPACITY.
 */
fly_status fly_model_draft_workspace_bytes(const fly_model_desc* desc, int32_t B, int32_t K,
                                           int32_t max_ctx_len, size_t* bytes);
fly_status fly_model_draft(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                           const int32_t* ctx, const int32_t* ctx_len, int32_t ctx_capacity,
                           int32_t max_ctx_len, int32_t B, int32_t K, int32_t* tokens, void* workspace,
                           size_t workspace_bytes, fly_stream stream);

/*
 * fly_decode_rounds with the draft model as drafter: every round drafts K tokens
 * with fly_model_draft, verifies them with the target (forward, row statistics,
 * loose acceptance) and rolls the sequences and the target's cache forward.
 * The two models must share the vocabulary.  Bounds as for fly_decode_rounds,
 * plus draft_kv->capacity >= seq->max_ctx_len + rounds*(K+1) + K.
 * Workspace: fly_decode_model_workspace_bytes(desc, draft_desc, B, K, kv->max_kv_len + rounds*(K+1)).
 */
fly_status fly_decode_model_workspace_bytes(const fly_model_desc* desc, const fly_model_desc* draft_desc,
                                            int32_t B, int32_t K, int32_t max_kv_len_end, size_t* bytes);
fly_status fly_decode_rounds_model(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                                   const fly_model_desc* draft_desc, const fly_weights* draft_w,
                                   const fly_kv_cache* draft_kv, const fly_sequences* seq,
                                   const float* row_scale, int32_t B, int32_t K, float theta, int32_t W,
                                   int32_t rounds, void* workspace, size_t workspace_bytes,
                                   fly_stream stream);

/*
 * Decoder layers [layer_begin, layer_end) applied in place to a residual
 * stream x [device] fp32 [M, d] (the middle of fly_verify_block, exposed for
 * per-layer checks and per-layer timing).  Uses the same workspace.
 */
fly_status fly_decoder_layers(const fly_model_desc* desc, const fly_weights* w,
                              const fly_kv_cache* kv, float* x, int32_t layer_begin,
                              int32_t layer_end, int32_t B, int32_t K, void* workspace,
                              size_t workspace_bytes, fly_stream stream);

/*
 * LM head with fused row statistics (Eq. 1 and Eq. 5).
 *   hidden  [device] [M, d] in the model dtype (already normalised)
 *   w_lm    [device] packed [d, V]
 * Outputs [device]: argmax int32 [M] (lowest index on ties), p_top1 float [M],
 * h_norm float [M] = H / ln V, lse float [M] (nullable).
 * V must be a multiple of 16; d a multiple of 32 for FLY_BF16.
 */
fly_status fly_lmhead_entropy_argmax(const void* hidden, const void* w_lm, const float* row_scale,
                                     int32_t M, int32_t d, int32_t V, int32_t dtype,
                                     int32_t* argmax, float* p_top1, float* h_norm, float* lse,
                                     void* workspace, size_t workspace_bytes, fly_stream stream);

/*
 * The same with one token per row drawn from softmax(row_scale[m] * logits[m])
 * as well (see fly_verify_block_sampled for the construction; row m of this
 * call is row m of the counter).  sampled [device] int32 [M].  Same workspace.
 */
fly_status fly_lmhead_entropy_sample(const void* hidden, const void* w_lm, const float* row_scale,
                                     int32_t M, int32_t d, int32_t V, int32_t dtype, uint64_t seed,
                                     uint64_t offset, int32_t* sampled, int32_t* argmax, float* p_top1,
                                     float* h_norm, float* lse, void* workspace, size_t workspace_bytes,
                                     fly_stream stream);

/*
 * fly_lmhead_entropy_argmax for callers that cannot allocate device memory or
 * pass a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments without the workspace, same
 * kernels, same results bit for bit.  The partial row statistics live in a
 * 16 MiB array that is part of the library's device image (every GPU the library
 * runs on holds its own copy until the process ends); the call allocates and
 * frees nothing.  A request whose fly_lmhead_workspace_bytes exceeds 16 MiB
 * (about 170 rows at a 128256-token vocabulary) returns FLY_ERR_STATIC_SCRATCH
 * with nothing launched.  All calls on one GPU share the array: calls that
 * overlap on one GPU (different streams, different threads) race and must be
 * serialised by the caller; calls on one stream are safe back to back.
 */
#define FLY_LMHEAD_STATIC_SCRATCH_BYTES (16u << 20)
fly_status fly_lmhead_entropy_argmax_static(const void* hidden, const void* w_lm, const float* row_scale,
                                            int32_t M, int32_t d, int32_t V, int32_t dtype,
                                            int32_t* argmax, float* p_top1, float* h_norm, float* lse,
                                            fly_stream stream);

/*
 * FLy's loose acceptance rule (Eqs. 2-11; Algorithm 1 steps 3-4).
 *   draft       [device] int32 [B, K]      draft_1..draft_K
 *   tgt_argmax  [device] int32 [B, K+1]    y_1..y_{K+1}
 *   h_norm      [device] float [B, K+1]    h_1..h_{K+1} (the last is unused)
 * A mismatch at j is rejected when h_j < theta, when j + W > K, or when any
 * of positions j+1..j+W mismatches; s is the first rejected position, or K+1.
 * Outputs [device]: accept_len[b] = s-1, next_token[b] = y_s, n_loose[b]
 * (nullable) = number of mismatching drafts among the kept ones.
 * 1 <= K <= 63, W >= 0, theta not NaN (theta > 1 gives exact-match decoding).
 */
fly_status fly_accept(const int32_t* draft, const int32_t* tgt_argmax, const float* h_norm,
                      int32_t B, int32_t K, float theta, int32_t W, int32_t* accept_len,
                      int32_t* next_token, int32_t* n_loose, fly_stream stream);

/*
 * A plain projection as the layers run it (q/k/v, output and down projections;
 * exposed for per-kernel timing and checks): split-K partial sums
 *   partial[s, m, n] = sum over the k-range of split s of xn[m, k] * W[k, n]
 *   xn       [device] [M, Kd] model dtype;  w [device] packed [Kd, N]
 *   partial  [device] float [splits, M, N]; partial_bytes is its size, at least
 *            16*M*N*4 is always enough; *splits_out [host] receives the split count
 */
fly_status fly_proj_partial(const void* xn, const void* w, float* partial, int32_t M, int32_t N,
                            int32_t Kd, int32_t dtype, int32_t* splits_out, size_t partial_bytes,
                            fly_stream stream);

/*
 * Gate/up projection with the SwiGLU product fused into the GEMM epilogue
 * (the widest GEMM of a layer; exposed for per-kernel timing and checks):
 *   a[m, f] = silu(xn[m] . Wg[:, f]) * (xn[m] . Wu[:, f])
 *   xn        [device] [M, d] model dtype
 *   w_gateup  [device] packed [d, 2F], 16-column tiles alternating gate / up
 *   a         [device] [M, F] model dtype
 */
fly_status fly_gateup_swiglu(const void* xn, const void* w_gateup, void* a, int32_t M, int32_t d,
                             int32_t F, int32_t dtype, fly_stream stream);

/*
 * (K+1)-query causal grouped-query attention against the cache of one layer
 * (exposed for the long-cache workload and for per-kernel timing).
 *   q  [device] [M, Hq*hd] model dtype, already rotated
 *   o  [device] [M, Hq*hd] model dtype
 * Reads cache rows 0..kv_len[b]+i for query i; the K+1 new rows must already
 * be in the cache.  Workspace as for fly_verify_block.
 */
fly_status fly_attention(const fly_model_desc* desc, const fly_kv_cache* kv, int32_t layer,
                         const void* q, void* o, int32_t B, int32_t K, void* workspace,
                         size_t workspace_bytes, fly_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* FLY_H */
