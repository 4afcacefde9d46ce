// C ABI of the FLy verification step: argument validation, workspace
// planning and the launch sequence.  See include/fly.h for the contract.
#include <math.h>
#include <atomic>
#include <stdlib.h>
#include <string.h>

#include "fly_common.h"

namespace {

// --- tuning knobs (0 = automatic); set through fly_set_tuning.  Atomics: a change from one thread
// while another plans a call is seen by that call or by the next, never torn. ---------------
std::atomic<int> g_force_nt{0};
std::atomic<int> g_force_splits{0};
std::atomic<int> g_target_wgs{256};
std::atomic<int> g_mt_max{9};
std::atomic<int> g_tiled{0};  // 0 automatic, 1 never, 2, 3, 4 or 6: always, with that workgroup shape
std::atomic<int> g_wide{0};   // 0 automatic (81..256 rows), 1 never, 3, 4, 5, 6 or 8: always, with that many 32-row tiles

inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline size_t elem_size(int dtype) { return dtype == FLY_BF16 ? 2 : 4; }

int pick_mt(int rows) {
  int tiles = (rows + 15) / 16;
  const int opts[5] = {1, 2, 3, 5, 9};
  for (int i = 0; i < 5; ++i)
    if (tiles <= opts[i]) return opts[i];
  return 9;
}

// Plan of one bf16 GEMM.  Measured on MI355X: the kernel streams best with
// about one workgroup per compute unit (256), each wave holding as many column
// strips as the register file allows (4 for up to 48 rows, else 2), so that
// roughly 128 KiB of weight loads are in flight per compute unit.  Narrow
// outputs reach that workgroup count by split-K with two-strip waves (measured
// at the 8B and 70B projection shapes: never slower than four-strip waves with
// twice the splits, and they write half the partial sums).  A split shorter
// than twenty 128-wide chunks spends much of its time filling the register ring:
// then one split fewer wins even though fewer compute units are busy (output
// projection at 70B width: 3 x 64 workgroups beat 4 x 64).
int splits_for(int nblocks, int nchunks) {
  int s = (g_target_wgs + nblocks / 2) / nblocks;  // round to nearest
  if (s > 2 && (nchunks + s - 1) / s < 20) s -= 1;
  int max_splits = nchunks / 4;                     // at least four 128-wide chunks per split
  if (max_splits < 1) max_splits = 1;
  if (s > max_splits) s = max_splits;
  if (s > 16) s = 16;
  if (s < 1) s = 1;
  int cps = (nchunks + s - 1) / s;                  // drop empty trailing splits
  return (nchunks + cps - 1) / cps;
}

// Above 128 rows the LDS-tiled kernel takes over (measured: already at 136 rows
// its 192-row workgroups beat the streaming kernel's nine 16-row tiles per wave).  Its workgroups cover 128, 192,
// 256 or 384 rows: the shape that pads M least wins, the larger one on a tie (fewer
// bytes staged per flop).
// Split-K factor of the two kernels that take one workgroup per compute unit (LDS-tiled, wide).
// `wgs` workgroups per split, `steps` pipeline steps along k.  The launch runs in
// ceil(wgs * s / target) rounds of workgroups of steps / s steps each, and a round that is
// not full takes as long as a full one: 288 workgroups on 256 units are two rounds.  Every
// split also writes and re-reads a block of fp32 partial sums (about 5% per split,
// measured at the 405B and 70B widths).  At least sixteen steps per split.
static int pick_splits(int wgs, int steps) {
  if (g_force_splits) return g_force_splits;
  int best = 1;
  double best_cost = 0.0;
  for (int sp = 1; sp <= 16; ++sp) {
    if (sp > 1 && steps / sp < 16) break;
    const int per = (steps + sp - 1) / sp;
    const int rounds = (wgs * sp + g_target_wgs - 1) / g_target_wgs;
    const double cost = (double)rounds * per * (1.0 + 0.05 * sp);
    if (sp == 1 || cost < best_cost) {
      best = sp;
      best_cost = cost;
    }
  }
  return best;
}

GemmPlan plan_gemm_tiled(int M, int N, int Kd, bool allow_split, int forced) {
  GemmPlan p{1, 1, 1, 1, 3, 0};
  auto padded = [&](int shape) {
    const int rows = gemm_bf16_tiled_rows(shape);
    return (M + rows - 1) / rows * rows;
  };
  if (forced) {
    p.tiled = forced;
  } else {
    p.tiled = 2;
    if (padded(3) <= padded(p.tiled)) p.tiled = 3;
    if (padded(4) <= padded(p.tiled)) p.tiled = 4;
    if (padded(6) <= padded(p.tiled)) p.tiled = 6;
  }
  p.mblocks = padded(p.tiled) / gemm_bf16_tiled_rows(p.tiled);
  if (allow_split) {
    const int cols = gemm_bf16_tiled_cols(p.tiled);
    const int wgs = (N + cols - 1) / cols * p.mblocks;
    const int ktiles = Kd / 32;
    int s = pick_splits(wgs, ktiles);
    int max_splits = ktiles / 16;  // at least sixteen k-steps per split (also for a forced factor)
    if (s > max_splits) s = max_splits;
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    int kps = (ktiles + s - 1) / s;
    p.splits = (ktiles + kps - 1) / kps;
  }
  return p;
}

// 81..256 rows: the weight-streaming kernel with 32 x 32 tiles, one workgroup per
// 256 columns.  Narrow outputs reach one workgroup per compute unit by split-K
// with at least sixteen 64-wide chunks per split.
GemmPlan plan_gemm_wide(int M, int N, int Kd, bool allow_split, int forced) {
  GemmPlan p{1, 1, 1, 1, 0, 0};
  p.wide = forced ? forced : M <= 96 ? 3 : M <= 128 ? 4 : M <= 160 ? 5 : M <= 192 ? 6 : 8;
  if (allow_split) {
    const int cols = gemm_bf16_wide_cols();
    const int wgs = (N + cols - 1) / cols;
    const int nchunks = (Kd / 32 + 1) / 2;
    int s = pick_splits(wgs, nchunks);
    int max_splits = nchunks / 16;
    if (s > max_splits) s = max_splits;
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    const int cps = (nchunks + s - 1) / s;  // drop empty trailing splits
    p.splits = (nchunks + cps - 1) / cps;
  }
  return p;
}

GemmPlan plan_gemm(int M, int N, int Kd, bool allow_split, bool need_even_nt) {
  // Measured at the 70B width for 36..160 rows and at the 405B-slice (136 rows) and 70B batch-16
  // (256 rows) shapes: up to 80 rows the kernel with 16-row tiles wins, from 81 to 256 rows the
  // wide kernel wins or ties for every GEMM of the layer and for the LM head.
  if (g_wide >= 3 || (g_wide == 0 && g_tiled < 2 && M > 80 && M <= 256))
    return plan_gemm_wide(M, N, Kd, allow_split, g_wide >= 3 ? g_wide.load() : 0);
  if (g_tiled >= 2 || (g_tiled == 0 && M > 128)) return plan_gemm_tiled(M, N, Kd, allow_split, g_tiled);
  GemmPlan p;
  p.tiled = 0;
  p.wide = 0;
  const int rows_max = g_mt_max * 16;
  p.mblocks = (M + rows_max - 1) / rows_max;
  p.mt = p.mblocks > 1 ? g_mt_max.load() : pick_mt(M);
  const int ntiles = N / 16;
  const int nchunks = (Kd / 32 + 3) / 4;
  const int nt_max = 4;
  int nt = nt_max;
  auto blocks = [&](int t) { return (ntiles + 4 * t - 1) / (4 * t); };
  if (g_force_nt) {
    nt = g_force_nt;
  } else if (allow_split) {
    nt = 2;
  } else {
    // no split-K possible: narrow the wave tile until the launch has enough workgroups
    while (nt > 1 && blocks(nt) < g_target_wgs * 3 / 4) nt /= 2;
  }
  if (nt > nt_max) nt = nt_max;
  if (need_even_nt && nt < 2) nt = 2;
  p.nt = nt;
  p.splits = 1;
  if (allow_split) p.splits = g_force_splits ? g_force_splits.load() : splits_for(blocks(nt), nchunks);
  if (allow_split && g_force_splits) {
    int cps = (nchunks + p.splits - 1) / p.splits;
    p.splits = (nchunks + cps - 1) / cps;
  }
  return p;
}

struct Workspace {
  float* x;          // [M, d] residual stream
  void* xn;          // [M, d] normalised activations (model dtype)
  float* partial;    // split-K partial sums
  void* q;           // [M, Hq*hd]
  void* o;           // [M, Hq*hd]
  void* a;           // [M, F]
  float* rope;       // [M, hd/2, 2]
  float* attn;       // attention split partials
  float* lm_partial; // LM-head statistics partials
  size_t bytes;
};

struct Plans {
  GemmPlan qkv, wo, gateup, down, lm;
  AttnPlan attn;
  int lm_parts;
};

// Per (row, part): four floats of softmax statistics, then (behind all of them) two floats of the
// sampled-token pick.
size_t lmhead_partial_floats(int M, int V, int dtype, const GemmPlan& lm) {
  int parts = dtype == FLY_BF16 ? gemm_bf16_lmhead_parts(V, lm) : gemm_f32_lmhead_parts(V);
  return (size_t)M * parts * 6;
}

fly_status check_desc(const fly_model_desc* desc) {
  if (!desc) return FLY_ERR_NULL_POINTER;
  if (desc->dtype != FLY_F32 && desc->dtype != FLY_BF16) return FLY_ERR_DTYPE;
  if (desc->n_layers < 0 || desc->d < 16 || desc->n_q_heads < 1 || desc->n_kv_heads < 1 ||
      desc->ffn < 16 || desc->vocab < 16)
    return FLY_ERR_BAD_SHAPE;
  if (desc->n_q_heads % desc->n_kv_heads != 0) return FLY_ERR_BAD_SHAPE;
  if (desc->dtype == FLY_BF16) {
    if (desc->head_dim != 128) return FLY_ERR_HEAD_DIM;
    if (desc->d % 32 != 0 || desc->ffn % 32 != 0 || desc->vocab % 16 != 0) return FLY_ERR_BAD_SHAPE;
  } else {
    if (desc->head_dim != 64 && desc->head_dim != 128) return FLY_ERR_HEAD_DIM;
    if (desc->d % 16 != 0 || desc->ffn % 16 != 0 || desc->vocab % 16 != 0) return FLY_ERR_BAD_SHAPE;
  }
  return FLY_OK;
}

fly_status check_block(int B, int K) {
  // at most 65536 sequences: row and table indices (B * (K+1) * head_dim / 2 ...) stay far inside int32
  if (B < 1 || B > (1 << 16)) return FLY_ERR_BAD_SHAPE;
  if (K < 1 || K > 63) return FLY_ERR_K_RANGE;
  return FLY_OK;
}

fly_status make_plans(const fly_model_desc* desc, int B, int K, int max_kv_len, Plans* pl) {
  const int M = B * (K + 1);
  const int qkvN = (desc->n_q_heads + 2 * desc->n_kv_heads) * desc->head_dim;
  const int qdim = desc->n_q_heads * desc->head_dim;
  if (desc->dtype == FLY_BF16) {
    pl->qkv = plan_gemm(M, qkvN, desc->d, true, false);
    pl->wo = plan_gemm(M, desc->d, qdim, true, false);
    pl->gateup = plan_gemm(M, 2 * desc->ffn, desc->d, false, true);
    pl->down = plan_gemm(M, desc->d, desc->ffn, true, false);
    pl->lm = plan_gemm(M, desc->vocab, desc->d, false, false);
    pl->attn = plan_attention(B, K, desc->n_q_heads, desc->n_kv_heads, max_kv_len + K + 1);
    if (pl->attn.qblocks > 16) return FLY_ERR_BAD_SHAPE;  // more than 4096 query rows per KV head
  } else {
    GemmPlan one{1, 1, 1, 1};
    pl->qkv = pl->wo = pl->gateup = pl->down = pl->lm = one;
    pl->attn = AttnPlan{1, 64, 1, 1};
  }
  pl->lm_parts = desc->dtype == FLY_BF16 ? gemm_bf16_lmhead_parts(desc->vocab, pl->lm)
                                         : gemm_f32_lmhead_parts(desc->vocab);
  return FLY_OK;
}

// Carve the workspace; with base == NULL only the size is computed.
void carve(const fly_model_desc* desc, int B, int K, const Plans& pl, void* base, Workspace* ws) {
  const size_t M = (size_t)B * (K + 1);
  const size_t es = elem_size(desc->dtype);
  const size_t qkvN = (size_t)(desc->n_q_heads + 2 * desc->n_kv_heads) * desc->head_dim;
  const size_t qdim = (size_t)desc->n_q_heads * desc->head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void* p = base ? (void*)((char*)base + off) : nullptr;
    off += round_up(bytes, 256);
    return p;
  };
  ws->x = (float*)take(M * desc->d * 4);
  ws->xn = take(M * desc->d * es);
  size_t pf = (size_t)pl.qkv.splits * M * qkvN;
  size_t pf2 = (size_t)pl.wo.splits * M * desc->d;
  size_t pf3 = (size_t)pl.down.splits * M * desc->d;
  if (pf2 > pf) pf = pf2;
  if (pf3 > pf) pf = pf3;
  ws->partial = (float*)take(pf * 4);
  ws->q = take(M * qdim * es);
  ws->o = take(M * qdim * es);
  ws->a = take(M * (size_t)desc->ffn * es);
  ws->rope = (float*)take(M * desc->head_dim * 4);
  size_t af = desc->dtype == FLY_BF16 ? attention_workspace_floats(B, K, desc->n_q_heads, desc->n_kv_heads,
                                                                   desc->head_dim, pl.attn)
                                      : 0;
  ws->attn = (float*)take(af * 4);
  ws->lm_partial = (float*)take((size_t)M * pl.lm_parts * 24);  // statistics, then picks
  ws->bytes = off;
}

#define HIP_TRY(expr)                          \
  do {                                         \
    hipError_t _e = (expr);                    \
    if (_e != hipSuccess) return FLY_ERR_LAUNCH; \
  } while (0)

fly_status check_kv(const fly_model_desc* desc, const fly_kv_cache* kv, int K, int layer_begin,
                    int layer_end) {
  if (!kv || !kv->kv_len) return FLY_ERR_NULL_POINTER;
  if (layer_end > layer_begin && (!kv->k_layers || !kv->v_layers)) return FLY_ERR_NULL_POINTER;
  if (kv->capacity < 64 || kv->capacity % 64 != 0) return FLY_ERR_BAD_SHAPE;
  if (kv->max_kv_len < 0) return FLY_ERR_BAD_SHAPE;
  if ((int64_t)kv->max_kv_len + K + 1 > kv->capacity) return FLY_ERR_KV_CAPACITY;
  for (int l = layer_begin; l < layer_end; ++l) {
    if (!kv->k_layers[l] || !kv->v_layers[l]) return FLY_ERR_NULL_POINTER;
    if (!aligned16(kv->k_layers[l]) || !aligned16(kv->v_layers[l])) return FLY_ERR_ALIGNMENT;
  }
  return FLY_OK;
}

fly_status check_weights(const fly_model_desc* desc, const fly_weights* w, int layer_begin,
                         int layer_end, bool need_head) {
  if (!w) return FLY_ERR_NULL_POINTER;
  if (layer_end > layer_begin && !w->layers) return FLY_ERR_NULL_POINTER;
  for (int l = layer_begin; l < layer_end; ++l) {
    const fly_layer_weights& lw = w->layers[l];
    const void* ps[6] = {lw.w_qkv, lw.w_o, lw.w_gateup, lw.w_down, lw.g_attn, lw.g_ffn};
    for (int i = 0; i < 6; ++i) {
      if (!ps[i]) return FLY_ERR_NULL_POINTER;
      if (!aligned16(ps[i])) return FLY_ERR_ALIGNMENT;
    }
  }
  if (layer_end > layer_begin) {
    // the norm after the last requested layer uses the next layer's gain (or g_final)
    const void* next_gain = layer_end < desc->n_layers ? w->layers[layer_end].g_attn : w->g_final;
    if (!next_gain) return FLY_ERR_NULL_POINTER;
    if (!aligned16(next_gain)) return FLY_ERR_ALIGNMENT;
  }
  if (need_head) {
    if (!w->embed || !w->g_final || !w->w_lm) return FLY_ERR_NULL_POINTER;
    if (!aligned16(w->embed) || !aligned16(w->g_final) || !aligned16(w->w_lm)) return FLY_ERR_ALIGNMENT;
  }
  return FLY_OK;
}

#define FLY_TRY(expr)               \
  do {                              \
    fly_status _s = (expr);         \
    if (_s != FLY_OK) return _s;    \
  } while (0)

// One GEMM of the layer in either dtype; bf16 may leave split-K partials.
fly_status run_gemm(int dtype, const void* X, const void* W, void* out, const float* row_scale, int M,
                    int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st,
                    const LmSample& smp = LmSample{}) {
  if (dtype == FLY_BF16)
    HIP_TRY(launch_gemm_bf16((const bf16_t*)X, (const bf16_t*)W, out, row_scale, M, N, Kd, plan, epi, st, smp));
  else
    HIP_TRY(launch_gemm_f32((const float*)X, (const float*)W, out, row_scale, M, N, Kd, epi, st, smp));
  return FLY_OK;
}

// A request to draw the row's token as well (seed, offset, where the drawn tokens go).
struct SampleRequest {
  uint64_t seed, offset;
  int32_t* sampled;  // [M]
};
// LM head with fused statistics on `partial` (M * parts * 6 floats): logits stay in registers.
fly_status run_lmhead(int dtype, const void* xn, const void* w_lm, float* partial, const float* row_scale,
                      int M, int V, int d, const GemmPlan& lm, int parts, int32_t* argmax, float* p_top1,
                      float* h_norm, float* lse, const SampleRequest* sr, hipStream_t st) {
  if (sr == nullptr) {
    FLY_TRY(run_gemm(dtype, xn, w_lm, partial, row_scale, M, V, d, lm, EPI_LMHEAD, st));
    HIP_TRY(launch_lmhead_combine(partial, parts, M, V, argmax, p_top1, h_norm, lse, st));
    return FLY_OK;
  }
  LmSample smp;
  smp.pick = partial + (size_t)M * parts * 4;
  smp.key0 = (uint32_t)sr->seed;
  smp.key1 = (uint32_t)(sr->seed >> 32);
  smp.ctr2 = (uint32_t)sr->offset;
  smp.ctr3 = (uint32_t)(sr->offset >> 32);
  FLY_TRY(run_gemm(dtype, xn, w_lm, partial, row_scale, M, V, d, lm, EPI_LMSAMPLE, st, smp));
  HIP_TRY(launch_lmhead_combine(partial, parts, M, V, argmax, p_top1, h_norm, lse, st, smp.pick, sr->sampled));
  return FLY_OK;
}

// Layers [l0, l1) on the residual stream ws.x; ws.xn must hold
// rmsnorm(x) * g_attn[l0] on entry and holds rmsnorm(x) * next_gain on exit
// (next_gain = g_attn of layer l1, or g_final after the last layer).
fly_status run_layers(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                      const Workspace& ws, const Plans& pl, int l0, int l1, int B, int K,
                      hipStream_t st) {
  const int M = B * (K + 1), d = desc->d, dt = desc->dtype;
  const int Hq = desc->n_q_heads, Hkv = desc->n_kv_heads, hd = desc->head_dim;
  const int qkvN = (Hq + 2 * Hkv) * hd, qdim = Hq * hd;
  for (int l = l0; l < l1; ++l) {
    const fly_layer_weights& lw = w->layers[l];
    // q, k, v projection -> rotate -> append to the cache
    FLY_TRY(run_gemm(dt, ws.xn, lw.w_qkv, ws.partial, nullptr, M, qkvN, d, pl.qkv, EPI_PARTIAL, st));
    HIP_TRY(launch_qkv_epilogue(ws.partial, pl.qkv.splits, ws.rope, ws.q, kv->k_layers[l],
                                kv->v_layers[l], kv->kv_len, dt, B, K, Hq, Hkv, hd, kv->capacity, st));
    // attention over prefix + new rows
    if (dt == FLY_BF16)
      HIP_TRY(launch_attention_bf16((const bf16_t*)ws.q, (const bf16_t*)kv->k_layers[l],
                                    (const bf16_t*)kv->v_layers[l], kv->kv_len, (bf16_t*)ws.o, ws.attn,
                                    B, K, Hq, Hkv, hd, kv->capacity, pl.attn, st));
    else
      HIP_TRY(launch_attention_f32((const float*)ws.q, (const float*)kv->k_layers[l],
                                   (const float*)kv->v_layers[l], kv->kv_len, (float*)ws.o, B, K, Hq,
                                   Hkv, hd, kv->capacity, st));
    // output projection + residual, then the FFN norm
    FLY_TRY(run_gemm(dt, ws.o, lw.w_o, ws.partial, nullptr, M, d, qdim, pl.wo, EPI_PARTIAL, st));
    HIP_TRY(launch_reduce_residual_norm(ws.x, ws.partial, pl.wo.splits, lw.g_ffn, ws.xn, dt, M, d,
                                        desc->rms_eps, st));
    // SwiGLU FFN + residual, then the next norm
    FLY_TRY(run_gemm(dt, ws.xn, lw.w_gateup, ws.a, nullptr, M, 2 * desc->ffn, d, pl.gateup, EPI_SWIGLU, st));
    FLY_TRY(run_gemm(dt, ws.a, lw.w_down, ws.partial, nullptr, M, d, desc->ffn, pl.down, EPI_PARTIAL, st));
    const void* next_gain = (l + 1 < desc->n_layers) ? w->layers[l + 1].g_attn : w->g_final;
    HIP_TRY(launch_reduce_residual_norm(ws.x, ws.partial, pl.down.splits, next_gain, ws.xn, dt, M, d,
                                        desc->rms_eps, st));
  }
  return FLY_OK;
}

// The forward of the step on a carved workspace (arguments already validated): embedding, layers,
// final norm, LM head with fused statistics.  K = 0 (one position per sequence) is allowed here.
fly_status run_forward(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                       const int32_t* tokens, const float* row_scale, int B, int K, int32_t* argmax,
                       float* p_top1, float* h_norm, float* lse, float* hidden_out, const Workspace& ws,
                       const Plans& pl, hipStream_t st, const SampleRequest* sr = nullptr) {
  const int M = B * (K + 1), d = desc->d, dt = desc->dtype;
  HIP_TRY(launch_rope_table(kv->kv_len, ws.rope, B, K, desc->head_dim, desc->rope_theta, st));
  HIP_TRY(launch_embed(tokens, w->embed, dt, ws.x, M, d, desc->vocab, st));
  const void* first_gain = desc->n_layers > 0 ? w->layers[0].g_attn : w->g_final;
  HIP_TRY(launch_reduce_residual_norm(ws.x, nullptr, 0, first_gain, ws.xn, dt, M, d, desc->rms_eps, st));
  FLY_TRY(run_layers(desc, w, kv, ws, pl, 0, desc->n_layers, B, K, st));
  if (hidden_out)
    HIP_TRY(hipMemcpyAsync(hidden_out, ws.x, (size_t)M * d * 4, hipMemcpyDeviceToDevice, st));
  return run_lmhead(dt, ws.xn, w->w_lm, ws.lm_partial, row_scale, M, desc->vocab, d, pl.lm, pl.lm_parts,
                    argmax, p_top1, h_norm, lse, sr, st);
}

// The step itself: forward, then the acceptance rule on (draft, target token, h).  The target's
// token is the argmax (Eq. 1) or, with a sample request, the token drawn from the same softmax.
fly_status run_verify(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                      const int32_t* tokens, const float* row_scale, int B, int K, float theta, int W,
                      const fly_verify_out* out, const Workspace& ws, const Plans& pl, hipStream_t st,
                      const SampleRequest* sr = nullptr) {
  FLY_TRY(run_forward(desc, w, kv, tokens, row_scale, B, K, out->argmax, out->p_top1, out->h_norm, out->lse,
                      out->hidden_out, ws, pl, st, sr));
  HIP_TRY(launch_accept(tokens + 1, K + 1, sr ? sr->sampled : out->argmax, out->h_norm, kv->kv_len, B, K,
                        theta, W, out->accept_len, out->next_token, out->n_loose, out->kv_len_out, st));
  return FLY_OK;
}

// Buffers of the model drafter (behind its forward workspace).
struct DraftScratch {
  int32_t *tok2, *len_steps, *drafts, *argmax2;
  float *p_top1, *h_norm;
  size_t bytes;
};
void carve_draft(int B, int K, void* base, DraftScratch* ds) {
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void* p = base ? (void*)((char*)base + off) : nullptr;
    off += round_up(bytes, 256);
    return p;
  };
  ds->tok2 = (int32_t*)take((size_t)2 * B * 4);
  ds->len_steps = (int32_t*)take((size_t)K * B * 4);
  ds->drafts = (int32_t*)take((size_t)K * B * 4);
  ds->argmax2 = (int32_t*)take((size_t)2 * B * 4);
  ds->p_top1 = (float*)take((size_t)2 * B * 4);
  ds->h_norm = (float*)take((size_t)2 * B * 4);
  ds->bytes = off;
}

// The drafter's cache: layer pointers and capacity only (its lengths follow from the sequences).
fly_status check_draft_kv(const fly_model_desc* desc, const fly_kv_cache* kv, int64_t max_rows) {
  if (!kv) return FLY_ERR_NULL_POINTER;
  if (desc->n_layers > 0 && (!kv->k_layers || !kv->v_layers)) return FLY_ERR_NULL_POINTER;
  if (kv->capacity < 64 || kv->capacity % 64 != 0) return FLY_ERR_BAD_SHAPE;
  if (max_rows > kv->capacity) return FLY_ERR_KV_CAPACITY;
  for (int l = 0; l < desc->n_layers; ++l) {
    if (!kv->k_layers[l] || !kv->v_layers[l]) return FLY_ERR_NULL_POINTER;
    if (!aligned16(kv->k_layers[l]) || !aligned16(kv->v_layers[l])) return FLY_ERR_ALIGNMENT;
  }
  return FLY_OK;
}

// K greedy passes of the draft model on carved buffers (arguments already validated):
// pass 1 over the last two tokens of every sequence, passes 2..K over one draft each.
fly_status run_model_draft(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                           const int32_t* ctx, const int32_t* ctx_len, int ctx_capacity, int B, int K,
                           int32_t* tokens, const Workspace& ws2, const Plans& pl2, const Workspace& ws1,
                           const Plans& pl1, const DraftScratch& ds, hipStream_t st) {
  HIP_TRY(launch_draft_prepare(ctx, ctx_len, ctx_capacity, B, K, ds.tok2, ds.len_steps, st));
  fly_kv_cache kvs = *kv;
  kvs.kv_len = ds.len_steps;
  FLY_TRY(run_forward(desc, w, &kvs, ds.tok2, nullptr, B, 1, ds.argmax2, ds.p_top1, ds.h_norm, nullptr, nullptr,
                      ws2, pl2, st));
  HIP_TRY(launch_draft_pick(ds.argmax2, B, ds.drafts, st));
  for (int i = 2; i <= K; ++i) {
    kvs.kv_len = ds.len_steps + (int64_t)(i - 1) * B;
    FLY_TRY(run_forward(desc, w, &kvs, ds.drafts + (int64_t)(i - 2) * B, nullptr, B, 0,
                        ds.drafts + (int64_t)(i - 1) * B, ds.p_top1, ds.h_norm, nullptr, nullptr, ws1, pl1, st));
  }
  HIP_TRY(launch_draft_assemble(ds.tok2, ds.drafts, B, K, tokens, st));
  return FLY_OK;
}

// Plans and workspace of the drafter's two pass shapes (two rows / one row per sequence); the two
// workspaces occupy the same memory, the scratch follows.
struct DraftSetup {
  Plans pl2, pl1;
  Workspace ws2, ws1;
  DraftScratch ds;
  size_t bytes;
};
fly_status setup_draft(const fly_model_desc* desc, int B, int K, int max_kv_len, void* base, DraftSetup* s) {
  FLY_TRY(make_plans(desc, B, 1, max_kv_len, &s->pl2));
  FLY_TRY(make_plans(desc, B, 0, max_kv_len, &s->pl1));
  carve(desc, B, 1, s->pl2, base, &s->ws2);
  carve(desc, B, 0, s->pl1, base, &s->ws1);
  const size_t fwd = s->ws2.bytes > s->ws1.bytes ? s->ws2.bytes : s->ws1.bytes;
  carve_draft(B, K, base ? (char*)base + fwd : nullptr, &s->ds);
  s->bytes = fwd + s->ds.bytes;
  return FLY_OK;
}

// Per-round buffers of the decode loop (behind the verification workspace).
struct DecodeScratch {
  int32_t *tokens, *accept_len, *next_token, *kv_len_out, *argmax, *n_loose, *sampled;
  float *h_norm, *p_top1;
  size_t bytes;
};
void carve_decode(int B, int K, void* base, DecodeScratch* ds) {
  const size_t M = (size_t)B * (K + 1);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void* p = base ? (void*)((char*)base + off) : nullptr;
    off += round_up(bytes, 256);
    return p;
  };
  ds->tokens = (int32_t*)take(M * 4);
  ds->accept_len = (int32_t*)take((size_t)B * 4);
  ds->next_token = (int32_t*)take((size_t)B * 4);
  ds->kv_len_out = (int32_t*)take((size_t)B * 4);
  ds->n_loose = (int32_t*)take((size_t)B * 4);
  ds->argmax = (int32_t*)take(M * 4);
  ds->h_norm = (float*)take(M * 4);
  ds->p_top1 = (float*)take(M * 4);
  ds->sampled = (int32_t*)take(M * 4);
  ds->bytes = off;
}

// --- the LM head for callers that cannot allocate ----------------------------
// The partial row statistics of fly_lmhead_entropy_argmax_static live in this
// file-scope device array instead of a caller's workspace.  In host code the
// array's name is only a stand-in: its device address is looked up once per
// device (hipGetSymbolAddress, with that device current) and kept; kernels,
// copies and memsets get the looked-up pointer, never the name.
#define FLY_STATIC_SCRATCH_BYTES (16u << 20)
#define FLY_MAX_DEVICES 64
static __device__ __align__(256) unsigned char fly_static_scratch[FLY_STATIC_SCRATCH_BYTES];
static void* g_static_scratch_ptr[FLY_MAX_DEVICES];  // per device; NULL = not looked up yet

// Device address of the scratch array on the current device (no allocation).
static fly_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= FLY_MAX_DEVICES) return FLY_ERR_LAUNCH;
  void* p = __atomic_load_n(&g_static_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (p == nullptr) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(fly_static_scratch)) != hipSuccess || p == nullptr)
      return FLY_ERR_LAUNCH;
    // two threads racing here look up the same address: the store is idempotent
    __atomic_store_n(&g_static_scratch_ptr[dev], p, __ATOMIC_RELEASE);
  }
  *out = p;
  return FLY_OK;
}

}  // namespace

extern "C" {

const char* fly_strerror(fly_status s) {
  switch (s) {
    case FLY_OK: return "ok";
    case FLY_ERR_NULL_POINTER: return "a required pointer is NULL";
    case FLY_ERR_BAD_SHAPE: return "a size is out of range or not a multiple of the tile granularity";
    case FLY_ERR_K_RANGE: return "K must be in [1, 63]";
    case FLY_ERR_WINDOW: return "W must be >= 0";
    case FLY_ERR_THETA: return "theta is NaN";
    case FLY_ERR_DTYPE: return "unknown dtype";
    case FLY_ERR_HEAD_DIM: return "unsupported head_dim";
    case FLY_ERR_ALIGNMENT: return "a device pointer is not 16-byte aligned";
    case FLY_ERR_WORKSPACE: return "workspace missing or too small";
    case FLY_ERR_KV_CAPACITY: return "max_kv_len + K + 1 exceeds the KV cache capacity";
    case FLY_ERR_LAUNCH: return "the HIP runtime refused a launch";
    case FLY_ERR_STATIC_SCRATCH: return "the request needs more than the 16 MiB static scratch array";
  }
  return "unknown status";
}

// Tuning knobs for experiments: "gemm_nt" (1, 2, 4; 0 = automatic), "gemm_tiled", "gemm_wide",
// "gemm_splits" (0 = automatic), "target_wgs" (workgroups a launch aims for), "wide_phase" (81..256-row
// GEMM: 1 = half of the waves request their loads after multiplying, 2 = all before, 0 = automatic),
// "tiled_phase" (LDS-tiled GEMM: 1 = odd waves request their loads in mid-step, 2 = all first, 0 = automatic),
// "attn_phase" (attention: 1 = odd waves request their stage loads after multiplying, 2 = all first, 0 = automatic).
fly_status fly_set_tuning(const char* key, int32_t value) {
  if (!key) return FLY_ERR_NULL_POINTER;
  if (!strcmp(key, "gemm_nt")) {
    if (value != 0 && value != 1 && value != 2 && value != 4) return FLY_ERR_BAD_SHAPE;
    g_force_nt = value;
  } else if (!strcmp(key, "gemm_splits")) {
    if (value < 0 || value > 16) return FLY_ERR_BAD_SHAPE;
    g_force_splits = value;
  } else if (!strcmp(key, "attn_splits")) {
    if (value < 0 || value > 256) return FLY_ERR_BAD_SHAPE;
    g_attn_force_splits = value;
  } else if (!strcmp(key, "attn_block_tiles")) {
    if (value < 0 || value > 8) return FLY_ERR_BAD_SHAPE;
    g_attn_force_block_tiles = value;
  } else if (!strcmp(key, "gemm_mt_max")) {
    if (value != 5 && value != 9) return FLY_ERR_BAD_SHAPE;
    g_mt_max = value;
  } else if (!strcmp(key, "gemm_tiled")) {
    if (value != 0 && value != 1 && gemm_bf16_tiled_rows(value) == 0) return FLY_ERR_BAD_SHAPE;
    g_tiled = value;
  } else if (!strcmp(key, "gemm_wide")) {
    if (value != 0 && value != 1 && value != 3 && value != 4 && value != 5 && value != 6 && value != 8)
      return FLY_ERR_BAD_SHAPE;
    g_wide = value;
  } else if (!strcmp(key, "wide_phase")) {
    if (value < 0 || value > 2) return FLY_ERR_BAD_SHAPE;
    g_wide_phase = value;
  } else if (!strcmp(key, "tiled_phase")) {
    if (value < 0 || value > 2) return FLY_ERR_BAD_SHAPE;
    g_tiled_phase = value;
  } else if (!strcmp(key, "attn_phase")) {
    if (value < 0 || value > 2) return FLY_ERR_BAD_SHAPE;
    g_attn_phase = value;
  } else if (!strcmp(key, "target_wgs")) {
    if (value < 1) return FLY_ERR_BAD_SHAPE;
    g_target_wgs = value;
  } else {
    return FLY_ERR_BAD_SHAPE;
  }
  return FLY_OK;
}

fly_status fly_packed_weight_bytes(int64_t k_in, int64_t n_dst, int32_t dtype, size_t* bytes) {
  if (!bytes) return FLY_ERR_NULL_POINTER;
  if (dtype != FLY_F32 && dtype != FLY_BF16) return FLY_ERR_DTYPE;
  if (k_in < 1 || n_dst < 16 || n_dst % 16 != 0) return FLY_ERR_BAD_SHAPE;
  if (dtype == FLY_BF16 && k_in % 32 != 0) return FLY_ERR_BAD_SHAPE;
  *bytes = (size_t)k_in * (size_t)n_dst * elem_size(dtype);
  return FLY_OK;
}

fly_status fly_pack_weight(const void* src, int64_t k_in, int64_t n_src, int32_t dtype, void* dst,
                           int64_t n_dst, int64_t tile_offset, int64_t tile_stride,
                           fly_stream stream) {
  if (!src || !dst) return FLY_ERR_NULL_POINTER;
  if (dtype != FLY_F32 && dtype != FLY_BF16) return FLY_ERR_DTYPE;
  if (k_in < 1 || n_src < 16 || n_src % 16 != 0 || n_dst < 16 || n_dst % 16 != 0) return FLY_ERR_BAD_SHAPE;
  if (dtype == FLY_BF16 && k_in % 32 != 0) return FLY_ERR_BAD_SHAPE;
  if (tile_offset < 0 || tile_stride < 1) return FLY_ERR_BAD_SHAPE;
  // the last source tile must land inside the destination
  if (tile_offset + (n_src / 16 - 1) * tile_stride >= n_dst / 16) return FLY_ERR_BAD_SHAPE;
  if (!aligned16(src) || !aligned16(dst)) return FLY_ERR_ALIGNMENT;
  HIP_TRY(launch_pack_weight(src, k_in, n_src, dtype, dst, n_dst, tile_offset, tile_stride,
                             (hipStream_t)stream));
  return FLY_OK;
}

fly_status fly_workspace_bytes(const fly_model_desc* desc, int32_t B, int32_t K, int32_t max_kv_len,
                               size_t* bytes) {
  if (!bytes) return FLY_ERR_NULL_POINTER;
  FLY_TRY(check_desc(desc));
  FLY_TRY(check_block(B, K));
  if (max_kv_len < 0) return FLY_ERR_BAD_SHAPE;
  Plans pl;
  FLY_TRY(make_plans(desc, B, K, max_kv_len, &pl));
  Workspace ws;
  carve(desc, B, K, pl, nullptr, &ws);
  *bytes = ws.bytes;
  return FLY_OK;
}

fly_status fly_lmhead_workspace_bytes(int32_t M, int32_t d, int32_t V, int32_t dtype, size_t* bytes) {
  if (!bytes) return FLY_ERR_NULL_POINTER;
  if (dtype != FLY_F32 && dtype != FLY_BF16) return FLY_ERR_DTYPE;
  if (M < 1 || d < 16 || V < 16 || V % 16 != 0) return FLY_ERR_BAD_SHAPE;
  if (dtype == FLY_BF16 && d % 32 != 0) return FLY_ERR_BAD_SHAPE;
  GemmPlan lm = dtype == FLY_BF16 ? plan_gemm(M, V, d, false, false) : GemmPlan{1, 1, 1, 1};
  *bytes = round_up(lmhead_partial_floats(M, V, dtype, lm) * 4, 256);
  return FLY_OK;
}

static fly_status lmhead_entry(const void* hidden, const void* w_lm, const float* row_scale, int32_t M,
                               int32_t d, int32_t V, int32_t dtype, int32_t* argmax, float* p_top1,
                               float* h_norm, float* lse, const SampleRequest* sr, void* workspace,
                               size_t workspace_bytes, fly_stream stream) {
  if (!hidden || !w_lm || !argmax || !p_top1 || !h_norm) return FLY_ERR_NULL_POINTER;
  if (sr && !sr->sampled) return FLY_ERR_NULL_POINTER;
  size_t need = 0;
  FLY_TRY(fly_lmhead_workspace_bytes(M, d, V, dtype, &need));
  if (!workspace || workspace_bytes < need) return FLY_ERR_WORKSPACE;
  if (!aligned16(hidden) || !aligned16(w_lm) || !aligned16(workspace)) return FLY_ERR_ALIGNMENT;
  GemmPlan lm = dtype == FLY_BF16 ? plan_gemm(M, V, d, false, false) : GemmPlan{1, 1, 1, 1};
  int parts = dtype == FLY_BF16 ? gemm_bf16_lmhead_parts(V, lm) : gemm_f32_lmhead_parts(V);
  return run_lmhead(dtype, hidden, w_lm, (float*)workspace, row_scale, M, V, d, lm, parts, argmax, p_top1,
                    h_norm, lse, sr, (hipStream_t)stream);
}

fly_status fly_lmhead_entropy_argmax(const void* hidden, const void* w_lm, const float* row_scale,
                                     int32_t M, int32_t d, int32_t V, int32_t dtype, int32_t* argmax,
                                     float* p_top1, float* h_norm, float* lse, void* workspace,
                                     size_t workspace_bytes, fly_stream stream) {
  return lmhead_entry(hidden, w_lm, row_scale, M, d, V, dtype, argmax, p_top1, h_norm, lse, nullptr,
                      workspace, workspace_bytes, stream);
}

fly_status fly_lmhead_entropy_sample(const void* hidden, const void* w_lm, const float* row_scale,
                                     int32_t M, int32_t d, int32_t V, int32_t dtype, uint64_t seed,
                                     uint64_t offset, int32_t* sampled, int32_t* argmax, float* p_top1,
                                     float* h_norm, float* lse, void* workspace, size_t workspace_bytes,
                                     fly_stream stream) {
  SampleRequest sr{seed, offset, sampled};
  return lmhead_entry(hidden, w_lm, row_scale, M, d, V, dtype, argmax, p_top1, h_norm, lse, &sr, workspace,
                      workspace_bytes, stream);
}

fly_status fly_lmhead_entropy_argmax_static(const void* hidden, const void* w_lm, const float* row_scale,
                                            int32_t M, int32_t d, int32_t V, int32_t dtype,
                                            int32_t* argmax, float* p_top1, float* h_norm, float* lse,
                                            fly_stream stream) {
  // sizes first: nothing below touches the device before the request is known to fit
  size_t need = 0;
  FLY_TRY(fly_lmhead_workspace_bytes(M, d, V, dtype, &need));
  if (need > FLY_STATIC_SCRATCH_BYTES) return FLY_ERR_STATIC_SCRATCH;
  if (!hidden || !w_lm || !argmax || !p_top1 || !h_norm) return FLY_ERR_NULL_POINTER;
  if (!aligned16(hidden) || !aligned16(w_lm)) return FLY_ERR_ALIGNMENT;
  void* scratch = nullptr;
  FLY_TRY(static_scratch(&scratch));
  // every partial record the combine step reads is written by the GEMM of the same call, so the
  // array needs no clearing between calls
  return lmhead_entry(hidden, w_lm, row_scale, M, d, V, dtype, argmax, p_top1, h_norm, lse, nullptr, scratch,
                      FLY_STATIC_SCRATCH_BYTES, stream);
}

fly_status fly_accept(const int32_t* draft, const int32_t* tgt_argmax, const float* h_norm, int32_t B,
                      int32_t K, float theta, int32_t W, int32_t* accept_len, int32_t* next_token,
                      int32_t* n_loose, fly_stream stream) {
  if (!draft || !tgt_argmax || !h_norm || !accept_len || !next_token) return FLY_ERR_NULL_POINTER;
  FLY_TRY(check_block(B, K));
  if (W < 0) return FLY_ERR_WINDOW;
  if (theta != theta) return FLY_ERR_THETA;
  HIP_TRY(launch_accept(draft, K, tgt_argmax, h_norm, nullptr, B, K, theta, W, accept_len, next_token,
                        n_loose, nullptr, (hipStream_t)stream));
  return FLY_OK;
}

fly_status fly_decoder_layers(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                              float* x, int32_t layer_begin, int32_t layer_end, int32_t B, int32_t K,
                              void* workspace, size_t workspace_bytes, fly_stream stream) {
  FLY_TRY(check_desc(desc));
  FLY_TRY(check_block(B, K));
  if (!x) return FLY_ERR_NULL_POINTER;
  if (layer_begin < 0 || layer_end > desc->n_layers || layer_begin > layer_end) return FLY_ERR_BAD_SHAPE;
  FLY_TRY(check_weights(desc, w, layer_begin, layer_end, false));
  FLY_TRY(check_kv(desc, kv, K, layer_begin, layer_end));
  Plans pl;
  FLY_TRY(make_plans(desc, B, K, kv->max_kv_len, &pl));
  Workspace ws;
  carve(desc, B, K, pl, nullptr, &ws);
  if (!workspace || workspace_bytes < ws.bytes) return FLY_ERR_WORKSPACE;
  if (!aligned16(workspace) || !aligned16(x)) return FLY_ERR_ALIGNMENT;
  carve(desc, B, K, pl, workspace, &ws);
  if (layer_begin == layer_end) return FLY_OK;
  hipStream_t st = (hipStream_t)stream;
  const int M = B * (K + 1);
  HIP_TRY(hipMemcpyAsync(ws.x, x, (size_t)M * desc->d * 4, hipMemcpyDeviceToDevice, st));
  HIP_TRY(launch_rope_table(kv->kv_len, ws.rope, B, K, desc->head_dim, desc->rope_theta, st));
  HIP_TRY(launch_reduce_residual_norm(ws.x, nullptr, 0, w->layers[layer_begin].g_attn, ws.xn,
                                      desc->dtype, M, desc->d, desc->rms_eps, st));
  FLY_TRY(run_layers(desc, w, kv, ws, pl, layer_begin, layer_end, B, K, st));
  HIP_TRY(hipMemcpyAsync(x, ws.x, (size_t)M * desc->d * 4, hipMemcpyDeviceToDevice, st));
  return FLY_OK;
}

fly_status fly_attention(const fly_model_desc* desc, const fly_kv_cache* kv, int32_t layer, const void* q,
                         void* o, int32_t B, int32_t K, void* workspace, size_t workspace_bytes,
                         fly_stream stream) {
  FLY_TRY(check_desc(desc));
  FLY_TRY(check_block(B, K));
  if (!q || !o) return FLY_ERR_NULL_POINTER;
  if (layer < 0 || layer >= desc->n_layers) return FLY_ERR_BAD_SHAPE;
  FLY_TRY(check_kv(desc, kv, K, layer, layer + 1));
  Plans pl;
  FLY_TRY(make_plans(desc, B, K, kv->max_kv_len, &pl));
  Workspace ws;
  carve(desc, B, K, pl, nullptr, &ws);
  if (!workspace || workspace_bytes < ws.bytes) return FLY_ERR_WORKSPACE;
  if (!aligned16(workspace) || !aligned16(q) || !aligned16(o)) return FLY_ERR_ALIGNMENT;
  carve(desc, B, K, pl, workspace, &ws);
  hipStream_t st = (hipStream_t)stream;
  if (desc->dtype == FLY_BF16)
    HIP_TRY(launch_attention_bf16((const bf16_t*)q, (const bf16_t*)kv->k_layers[layer],
                                  (const bf16_t*)kv->v_layers[layer], kv->kv_len, (bf16_t*)o, ws.attn, B,
                                  K, desc->n_q_heads, desc->n_kv_heads, desc->head_dim, kv->capacity,
                                  pl.attn, st));
  else
    HIP_TRY(launch_attention_f32((const float*)q, (const float*)kv->k_layers[layer],
                                 (const float*)kv->v_layers[layer], kv->kv_len, (float*)o, B, K,
                                 desc->n_q_heads, desc->n_kv_heads, desc->head_dim, kv->capacity, st));
  return FLY_OK;
}

fly_status fly_proj_partial(const void* xn, const void* w, float* partial, int32_t M, int32_t N,
                            int32_t Kd, int32_t dtype, int32_t* splits_out, size_t partial_bytes,
                            fly_stream stream) {
  if (!xn || !w || !partial || !splits_out) return FLY_ERR_NULL_POINTER;
  if (dtype != FLY_F32 && dtype != FLY_BF16) return FLY_ERR_DTYPE;
  if (M < 1 || N < 16 || N % 16 != 0 || Kd < 16) return FLY_ERR_BAD_SHAPE;
  if (dtype == FLY_BF16 && Kd % 32 != 0) return FLY_ERR_BAD_SHAPE;
  if (!aligned16(xn) || !aligned16(w) || !aligned16(partial)) return FLY_ERR_ALIGNMENT;
  GemmPlan plan = dtype == FLY_BF16 ? plan_gemm(M, N, Kd, true, false) : GemmPlan{1, 1, 1, 1};
  if (partial_bytes < (size_t)plan.splits * M * N * 4) return FLY_ERR_WORKSPACE;
  *splits_out = plan.splits;
  return run_gemm(dtype, xn, w, partial, nullptr, M, N, Kd, plan, EPI_PARTIAL, (hipStream_t)stream);
}

fly_status fly_gateup_swiglu(const void* xn, const void* w_gateup, void* a, int32_t M, int32_t d,
                             int32_t F, int32_t dtype, fly_stream stream) {
  if (!xn || !w_gateup || !a) return FLY_ERR_NULL_POINTER;
  if (dtype != FLY_F32 && dtype != FLY_BF16) return FLY_ERR_DTYPE;
  if (M < 1 || d < 16 || F < 16 || F % 16 != 0) return FLY_ERR_BAD_SHAPE;
  if (dtype == FLY_BF16 && d % 32 != 0) return FLY_ERR_BAD_SHAPE;
  if (!aligned16(xn) || !aligned16(w_gateup) || !aligned16(a)) return FLY_ERR_ALIGNMENT;
  GemmPlan plan = dtype == FLY_BF16 ? plan_gemm(M, 2 * F, d, false, true) : GemmPlan{1, 1, 1, 1};
  return run_gemm(dtype, xn, w_gateup, a, nullptr, M, 2 * F, d, plan, EPI_SWIGLU, (hipStream_t)stream);
}

static fly_status verify_entry(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                               const int32_t* tokens, const float* row_scale, int32_t B, int32_t K,
                               float theta, int32_t W, const fly_verify_out* out, const SampleRequest* sr,
                               void* workspace, size_t workspace_bytes, fly_stream stream) {
  FLY_TRY(check_desc(desc));
  if (sr && !sr->sampled) return FLY_ERR_NULL_POINTER;
  FLY_TRY(check_block(B, K));
  if (W < 0) return FLY_ERR_WINDOW;
  if (theta != theta) return FLY_ERR_THETA;
  if (!tokens || !out) return FLY_ERR_NULL_POINTER;
  if (!out->accept_len || !out->next_token || !out->kv_len_out || !out->argmax || !out->h_norm ||
      !out->p_top1)
    return FLY_ERR_NULL_POINTER;
  FLY_TRY(check_weights(desc, w, 0, desc->n_layers, true));
  FLY_TRY(check_kv(desc, kv, K, 0, desc->n_layers));
  Plans pl;
  FLY_TRY(make_plans(desc, B, K, kv->max_kv_len, &pl));
  Workspace ws;
  carve(desc, B, K, pl, nullptr, &ws);
  if (!workspace || workspace_bytes < ws.bytes) return FLY_ERR_WORKSPACE;
  if (!aligned16(workspace)) return FLY_ERR_ALIGNMENT;
  carve(desc, B, K, pl, workspace, &ws);
  return run_verify(desc, w, kv, tokens, row_scale, B, K, theta, W, out, ws, pl, (hipStream_t)stream, sr);
}

fly_status fly_verify_block(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                            const int32_t* tokens, const float* row_scale, int32_t B, int32_t K,
                            float theta, int32_t W, const fly_verify_out* out, void* workspace,
                            size_t workspace_bytes, fly_stream stream) {
  return verify_entry(desc, w, kv, tokens, row_scale, B, K, theta, W, out, nullptr, workspace,
                      workspace_bytes, stream);
}

fly_status fly_verify_block_sampled(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                                    const int32_t* tokens, const float* row_scale, int32_t B, int32_t K,
                                    float theta, int32_t W, uint64_t seed, uint64_t offset,
                                    int32_t* sampled, const fly_verify_out* out, void* workspace,
                                    size_t workspace_bytes, fly_stream stream) {
  SampleRequest sr{seed, offset, sampled};
  return verify_entry(desc, w, kv, tokens, row_scale, B, K, theta, W, out, &sr, workspace, workspace_bytes,
                      stream);
}

fly_status fly_pld_draft(const int32_t* ctx, const int32_t* ctx_len, int32_t ctx_capacity, int32_t B,
                         int32_t K, int32_t ngram_max, int32_t* tokens, int32_t* ngram,
                         fly_stream stream) {
  if (!ctx || !ctx_len || !tokens) return FLY_ERR_NULL_POINTER;
  FLY_TRY(check_block(B, K));
  if (ctx_capacity < 1 || ngram_max < 1 || ngram_max > 64) return FLY_ERR_BAD_SHAPE;
  HIP_TRY(launch_pld_draft(ctx, ctx_len, ctx_capacity, B, K, ngram_max, tokens, ngram, (hipStream_t)stream));
  return FLY_OK;
}

fly_status fly_decode_workspace_bytes(const fly_model_desc* desc, int32_t B, int32_t K,
                                      int32_t max_kv_len_end, size_t* bytes) {
  if (!bytes) return FLY_ERR_NULL_POINTER;
  FLY_TRY(check_desc(desc));
  FLY_TRY(check_block(B, K));
  if (max_kv_len_end < 0) return FLY_ERR_BAD_SHAPE;
  Plans pl;
  FLY_TRY(make_plans(desc, B, K, max_kv_len_end, &pl));
  Workspace ws;
  carve(desc, B, K, pl, nullptr, &ws);
  DecodeScratch ds;
  carve_decode(B, K, nullptr, &ds);
  *bytes = ws.bytes + ds.bytes;
  return FLY_OK;
}

// draw: NULL for the greedy loop, else {seed, offset}: round r draws the target's tokens with offset + r.
static fly_status decode_rounds_entry(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                                      const fly_sequences* seq, const float* row_scale, int32_t B, int32_t K,
                                      float theta, int32_t W, int32_t ngram_max, int32_t rounds,
                                      const uint64_t* draw, void* workspace, size_t workspace_bytes,
                                      fly_stream stream) {
  FLY_TRY(check_desc(desc));
  FLY_TRY(check_block(B, K));
  if (W < 0) return FLY_ERR_WINDOW;
  if (theta != theta) return FLY_ERR_THETA;
  if (!seq || !seq->ctx || !seq->ctx_len || !seq->kv_len) return FLY_ERR_NULL_POINTER;
  if (rounds < 0 || ngram_max < 1 || ngram_max > 64 || seq->ctx_capacity < 1 || seq->max_ctx_len < 1)
    return FLY_ERR_BAD_SHAPE;
  FLY_TRY(check_weights(desc, w, 0, desc->n_layers, true));
  FLY_TRY(check_kv(desc, kv, K, 0, desc->n_layers));
  if (kv->kv_len != seq->kv_len) return FLY_ERR_BAD_SHAPE;
  const int64_t grow = (int64_t)rounds * (K + 1);
  if ((int64_t)kv->max_kv_len + grow > kv->capacity) return FLY_ERR_KV_CAPACITY;
  if ((int64_t)seq->max_ctx_len + grow > seq->ctx_capacity) return FLY_ERR_KV_CAPACITY;
  // one plan for the whole call, made for the longest cache the call can reach
  fly_kv_cache kvr = *kv;
  kvr.max_kv_len = kv->max_kv_len + (int32_t)(rounds > 0 ? grow - (K + 1) : 0);
  Plans pl;
  FLY_TRY(make_plans(desc, B, K, kv->max_kv_len + (int32_t)grow, &pl));
  Workspace ws;
  carve(desc, B, K, pl, nullptr, &ws);
  DecodeScratch ds;
  carve_decode(B, K, nullptr, &ds);
  if (!workspace || workspace_bytes < ws.bytes + ds.bytes) return FLY_ERR_WORKSPACE;
  if (!aligned16(workspace)) return FLY_ERR_ALIGNMENT;
  carve(desc, B, K, pl, workspace, &ws);
  carve_decode(B, K, (char*)workspace + ws.bytes, &ds);
  fly_verify_out out{ds.accept_len, ds.next_token, ds.kv_len_out, ds.argmax, ds.h_norm, ds.p_top1,
                     nullptr, ds.n_loose, nullptr};
  hipStream_t st = (hipStream_t)stream;
  for (int r = 0; r < rounds; ++r) {
    int32_t* ngram_row = seq->ngram_trace ? seq->ngram_trace + (int64_t)r * B : nullptr;
    int32_t* trace_row = seq->accept_trace ? seq->accept_trace + (int64_t)r * B : nullptr;
    HIP_TRY(launch_pld_draft(seq->ctx, seq->ctx_len, seq->ctx_capacity, B, K, ngram_max, ds.tokens,
                             ngram_row, st));
    SampleRequest sr{draw ? draw[0] : 0, draw ? draw[1] + (uint64_t)r : 0, ds.sampled};
    FLY_TRY(run_verify(desc, w, &kvr, ds.tokens, row_scale, B, K, theta, W, &out, ws, pl, st,
                       draw ? &sr : nullptr));
    HIP_TRY(launch_roll_forward(seq->ctx, seq->ctx_len, seq->kv_len, seq->ctx_capacity, B, K, ds.tokens,
                                ds.accept_len, ds.next_token, ds.kv_len_out, ds.n_loose,
                                seq->accepted_total, seq->rounds_done, seq->loose_total, trace_row, st));
  }
  return FLY_OK;
}

fly_status fly_decode_rounds(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                             const fly_sequences* seq, const float* row_scale, int32_t B, int32_t K,
                             float theta, int32_t W, int32_t ngram_max, int32_t rounds,
                             void* workspace, size_t workspace_bytes, fly_stream stream) {
  return decode_rounds_entry(desc, w, kv, seq, row_scale, B, K, theta, W, ngram_max, rounds, nullptr,
                             workspace, workspace_bytes, stream);
}

fly_status fly_decode_rounds_sampled(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                                     const fly_sequences* seq, const float* row_scale, int32_t B, int32_t K,
                                     float theta, int32_t W, int32_t ngram_max, int32_t rounds,
                                     uint64_t seed, uint64_t offset, void* workspace,
                                     size_t workspace_bytes, fly_stream stream) {
  const uint64_t draw[2] = {seed, offset};
  return decode_rounds_entry(desc, w, kv, seq, row_scale, B, K, theta, W, ngram_max, rounds, draw, workspace,
                             workspace_bytes, stream);
}

fly_status fly_model_draft_workspace_bytes(const fly_model_desc* desc, int32_t B, int32_t K,
                                           int32_t max_ctx_len, size_t* bytes) {
  if (!bytes) return FLY_ERR_NULL_POINTER;
  FLY_TRY(check_desc(desc));
  FLY_TRY(check_block(B, K));
  if (max_ctx_len < 2) return FLY_ERR_BAD_SHAPE;
  DraftSetup ds;
  FLY_TRY(setup_draft(desc, B, K, max_ctx_len + K, nullptr, &ds));
  *bytes = ds.bytes;
  return FLY_OK;
}

fly_status fly_model_draft(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                           const int32_t* ctx, const int32_t* ctx_len, int32_t ctx_capacity,
                           int32_t max_ctx_len, int32_t B, int32_t K, int32_t* tokens, void* workspace,
                           size_t workspace_bytes, fly_stream stream) {
  FLY_TRY(check_desc(desc));
  FLY_TRY(check_block(B, K));
  if (!ctx || !ctx_len || !tokens) return FLY_ERR_NULL_POINTER;
  if (max_ctx_len < 2 || max_ctx_len > ctx_capacity) return FLY_ERR_BAD_SHAPE;
  FLY_TRY(check_weights(desc, w, 0, desc->n_layers, true));
  FLY_TRY(check_draft_kv(desc, kv, (int64_t)max_ctx_len + K));
  DraftSetup ds;
  FLY_TRY(setup_draft(desc, B, K, max_ctx_len + K, nullptr, &ds));
  if (!workspace || workspace_bytes < ds.bytes) return FLY_ERR_WORKSPACE;
  if (!aligned16(workspace)) return FLY_ERR_ALIGNMENT;
  FLY_TRY(setup_draft(desc, B, K, max_ctx_len + K, workspace, &ds));
  return run_model_draft(desc, w, kv, ctx, ctx_len, ctx_capacity, B, K, tokens, ds.ws2, ds.pl2, ds.ws1, ds.pl1,
                         ds.ds, (hipStream_t)stream);
}

fly_status fly_decode_model_workspace_bytes(const fly_model_desc* desc, const fly_model_desc* draft_desc,
                                            int32_t B, int32_t K, int32_t max_kv_len_end, size_t* bytes) {
  if (!bytes) return FLY_ERR_NULL_POINTER;
  size_t target = 0, drafter = 0;
  FLY_TRY(fly_decode_workspace_bytes(desc, B, K, max_kv_len_end, &target));
  FLY_TRY(fly_model_draft_workspace_bytes(draft_desc, B, K, max_kv_len_end + 1, &drafter));
  *bytes = target + drafter;
  return FLY_OK;
}

fly_status fly_decode_rounds_model(const fly_model_desc* desc, const fly_weights* w, const fly_kv_cache* kv,
                                   const fly_model_desc* draft_desc, const fly_weights* draft_w,
                                   const fly_kv_cache* draft_kv, const fly_sequences* seq,
                                   const float* row_scale, int32_t B, int32_t K, float theta, int32_t W,
                                   int32_t rounds, void* workspace, size_t workspace_bytes,
                                   fly_stream stream) {
  FLY_TRY(check_desc(desc));
  FLY_TRY(check_desc(draft_desc));
  FLY_TRY(check_block(B, K));
  if (W < 0) return FLY_ERR_WINDOW;
  if (theta != theta) return FLY_ERR_THETA;
  if (!seq || !seq->ctx || !seq->ctx_len || !seq->kv_len) return FLY_ERR_NULL_POINTER;
  if (rounds < 0 || seq->ctx_capacity < 2 || seq->max_ctx_len < 2) return FLY_ERR_BAD_SHAPE;
  if (draft_desc->vocab != desc->vocab) return FLY_ERR_BAD_SHAPE;  // one token alphabet
  FLY_TRY(check_weights(desc, w, 0, desc->n_layers, true));
  FLY_TRY(check_weights(draft_desc, draft_w, 0, draft_desc->n_layers, true));
  FLY_TRY(check_kv(desc, kv, K, 0, desc->n_layers));
  if (kv->kv_len != seq->kv_len) return FLY_ERR_BAD_SHAPE;
  const int64_t grow = (int64_t)rounds * (K + 1);
  if ((int64_t)kv->max_kv_len + grow > kv->capacity) return FLY_ERR_KV_CAPACITY;
  if ((int64_t)seq->max_ctx_len + grow > seq->ctx_capacity) return FLY_ERR_KV_CAPACITY;
  const int max_ctx_end = seq->max_ctx_len + (int32_t)grow;
  FLY_TRY(check_draft_kv(draft_desc, draft_kv, (int64_t)max_ctx_end + K));
  fly_kv_cache kvr = *kv;
  kvr.max_kv_len = kv->max_kv_len + (int32_t)(rounds > 0 ? grow - (K + 1) : 0);
  Plans pl;
  FLY_TRY(make_plans(desc, B, K, kv->max_kv_len + (int32_t)grow, &pl));
  Workspace ws;
  carve(desc, B, K, pl, nullptr, &ws);
  DecodeScratch ds;
  carve_decode(B, K, nullptr, &ds);
  DraftSetup dr;
  FLY_TRY(setup_draft(draft_desc, B, K, max_ctx_end + K, nullptr, &dr));
  const size_t target_bytes = round_up(ws.bytes + ds.bytes, 256);
  if (!workspace || workspace_bytes < target_bytes + dr.bytes) return FLY_ERR_WORKSPACE;
  if (!aligned16(workspace)) return FLY_ERR_ALIGNMENT;
  carve(desc, B, K, pl, workspace, &ws);
  carve_decode(B, K, (char*)workspace + ws.bytes, &ds);
  FLY_TRY(setup_draft(draft_desc, B, K, max_ctx_end + K, (char*)workspace + target_bytes, &dr));
  fly_verify_out out{ds.accept_len, ds.next_token, ds.kv_len_out, ds.argmax, ds.h_norm, ds.p_top1,
                     nullptr, ds.n_loose, nullptr};
  hipStream_t st = (hipStream_t)stream;
  for (int r = 0; r < rounds; ++r) {
    int32_t* trace_row = seq->accept_trace ? seq->accept_trace + (int64_t)r * B : nullptr;
    FLY_TRY(run_model_draft(draft_desc, draft_w, draft_kv, seq->ctx, seq->ctx_len, seq->ctx_capacity, B, K,
                            ds.tokens, dr.ws2, dr.pl2, dr.ws1, dr.pl1, dr.ds, st));
    FLY_TRY(run_verify(desc, w, &kvr, ds.tokens, row_scale, B, K, theta, W, &out, ws, pl, st));
    HIP_TRY(launch_roll_forward(seq->ctx, seq->ctx_len, seq->kv_len, seq->ctx_capacity, B, K, ds.tokens,
                                ds.accept_len, ds.next_token, ds.kv_len_out, ds.n_loose,
                                seq->accepted_total, seq->rounds_done, seq->loose_total, trace_row, st));
  }
  return FLY_OK;
}

}  // extern "C"
