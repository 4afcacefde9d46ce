// Shared declarations of the HIP sources (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include "../../include/fly.h"

typedef uint16_t bf16_t;  // raw bf16 bits
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define FLY_WAVE 64

// fp32 -> bf16, round to nearest even (NaN not handled: inputs are finite).
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi) {
  return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
}

// Same rounding through the packed hardware conversion (v_cvt_pk_bf16_f32, RNE).
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ uint32_t pack_bf2_hw(float lo, float hi) {
  bf16x2_t v;
  v.x = (__bf16)lo;
  v.y = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}
// 2^x through the hardware transcendental (1 ulp; exact for integer x; 0 for -inf).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename T> struct Act;
template <> struct Act<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Act<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf2f(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f2bf(v); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, FLY_WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, FLY_WAVE));
  return v;
}

// Running softmax statistics of a set of logits: maximum m, s = sum e^(l-m),
// t = sum (l-m) e^(l-m), and the lowest index attaining m.  From them
// lse = m + ln s and the entropy H = ln s - t/s (Eq. 5 rearranged).
struct RowStat {
  float m, s, t;
  int32_t idx;
};
__device__ __forceinline__ RowStat stat_empty() { return RowStat{-INFINITY, 0.f, 0.f, 0x7fffffff}; }
__device__ __forceinline__ RowStat stat_merge(const RowStat& a, const RowStat& b) {
  RowStat r;
  if (b.s == 0.f) return a;
  if (a.s == 0.f) return b;
  r.m = fmaxf(a.m, b.m);
  float da = a.m - r.m, db = b.m - r.m;  // <= 0
  float ea = __expf(da), eb = __expf(db);
  r.s = a.s * ea + b.s * eb;
  r.t = (a.t + da * a.s) * ea + (b.t + db * b.s) * eb;
  r.idx = (a.m > b.m) ? a.idx : (b.m > a.m) ? b.idx : min(a.idx, b.idx);
  return r;
}
__device__ __forceinline__ RowStat stat_shfl_xor(const RowStat& a, int o) {
  RowStat r;
  r.m = __shfl_xor(a.m, o, FLY_WAVE);
  r.s = __shfl_xor(a.s, o, FLY_WAVE);
  r.t = __shfl_xor(a.t, o, FLY_WAVE);
  r.idx = __shfl_xor(a.idx, o, FLY_WAVE);
  return r;
}

typedef __attribute__((ext_vector_type(16))) float f32x16;
// Softmax statistics of the sixteen logits a lane holds of one 32 x 32 tile (columns
// n0 + 8 (r/4) + 4 hi + r%4 of one row), folded into the row's running statistics.
__device__ __forceinline__ void stat_update_tile32(RowStat& run, const f32x16& v, float sc, int n0, int hi,
                                                   int N) {
  float mx = -INFINITY;
  int idx = 0x7fffffff;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int n = n0 + 8 * (r >> 2) + 4 * hi + (r & 3);
    const float x = v[r] * sc;
    if (n < N && x > mx) {
      mx = x;
      idx = n;
    }
  }
  if (idx == 0x7fffffff) return;  // tile entirely past the last column
  RowStat st{mx, 0.f, 0.f, idx};
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int n = n0 + 8 * (r >> 2) + 4 * hi + (r & 3);
    if (n < N) {
      const float dlt = v[r] * sc - mx;
      const float e = __expf(dlt);
      st.s += e;
      st.t += dlt * e;
    }
  }
  run = stat_merge(run, st);
}

// ---- drawing a token from the softmax of the scaled logits -----------------
// The paper reports temperature-1 results (Tables 1-2) and states its rule with
// the argmax only (Eqs. 1-2); here the drawn token takes the argmax's place.
// Gumbel-max construction: argmax_v (l_v + G_v) with independent standard Gumbel
// variates G_v = -ln(-ln u_v) is distributed as softmax(l), and it needs the
// logits once, in any order, like the other row statistics.  u_v comes from
// Philox4x32 with ten rounds (Salmon et al., SC 2011): word v % 4 of the block
// with counter (v / 4, row, offset low, offset high) and key (seed low, seed
// high); u = (top 23 bits + 1/2) / 2^23 lies strictly inside (0, 1).
struct LmSample {
  float* pick;           // [M][nparts][2]: largest perturbed logit and its column (as int bits)
  uint32_t key0, key1;   // seed
  uint32_t ctr2, ctr3;   // the caller's 64-bit offset: tells calls with one seed apart
};
struct RowPick {
  float z;
  int32_t idx;
};
__device__ __forceinline__ RowPick pick_empty() { return RowPick{-INFINITY, 0x7fffffff}; }
__device__ __forceinline__ RowPick pick_merge(const RowPick& a, const RowPick& b) {
  return (a.z > b.z) ? a : (b.z > a.z) ? b : (a.idx < b.idx ? a : b);
}
__device__ __forceinline__ RowPick pick_shfl_xor(const RowPick& a, int o) {
  return RowPick{__shfl_xor(a.z, o, FLY_WAVE), __shfl_xor(a.idx, o, FLY_WAVE)};
}
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
  // kept as a loop: the epilogues call this once per four logits of up to 48 register tiles, and
  // unrolled ten-fold those bodies outgrow what the compiler is willing to unroll around them
#pragma unroll 1
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0;
    c1 = lo1;
    c2 = n2;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0;
  out[1] = c1;
  out[2] = c2;
  out[3] = c3;
}
__device__ __forceinline__ float gumbel_from_bits(uint32_t bits) {
  const float u = ((float)(bits >> 9) + 0.5f) * 1.1920928955078125e-07f;  // 2^-23; exact in fp32
  // the inner logarithm must be accurate relative to its result also for u next to 1 (the largest
  // variates, the ones that win); the outer one only to ~1e-6 absolute
  return -__logf(-logf(u));
}
// Folds the four scaled logits of columns col0 .. col0+3 (col0 a multiple of 4) of row `row`.
__device__ __forceinline__ void pick_update4(RowPick& p, float v0, float v1, float v2, float v3, int col0,
                                             int row, const LmSample& smp) {
  uint32_t x[4];
  philox4x32_10((uint32_t)col0 >> 2, (uint32_t)row, smp.ctr2, smp.ctr3, smp.key0, smp.key1, x);
  const float v[4] = {v0, v1, v2, v3};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float z = v[e] + gumbel_from_bits(x[e]);
    if (z > p.z || (z == p.z && col0 + e < p.idx)) {
      p.z = z;
      p.idx = col0 + e;
    }
  }
}
// The sixteen logits a lane holds of one 32 x 32 matrix-core tile (see stat_update_tile32) are
// four aligned groups of four columns.
__device__ __forceinline__ void pick_update_tile32(RowPick& p, const f32x16& v, float sc, int n0, int hi,
                                                   int N, int row, const LmSample& smp) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int col0 = n0 + 8 * q + 4 * hi;
    if (col0 < N)  // N is a multiple of 16: a group of four is inside or outside as a whole
      pick_update4(p, v[4 * q] * sc, v[4 * q + 1] * sc, v[4 * q + 2] * sc, v[4 * q + 3] * sc, col0, row, smp);
  }
}
// One column (the fp32 kernel holds one logit per lane).
__device__ __forceinline__ RowPick pick_one(float v, int col, int row, const LmSample& smp) {
  uint32_t x[4];
  philox4x32_10((uint32_t)col >> 2, (uint32_t)row, smp.ctr2, smp.ctr3, smp.key0, smp.key1, x);
  const uint32_t bits = (col & 3) == 0 ? x[0] : (col & 3) == 1 ? x[1] : (col & 3) == 2 ? x[2] : x[3];
  return RowPick{v + gumbel_from_bits(bits), col};
}
__device__ __forceinline__ void pick_store(const LmSample& smp, int64_t slot, const RowPick& p) {
  smp.pick[2 * slot] = p.z;
  smp.pick[2 * slot + 1] = __int_as_float(p.idx);
}

// LDS-direct load: every lane gives its own global address of 16 bytes, the wave's
// 1 KiB lands at lds_base + 16 * lane (lds_base wave-uniform, passed in M0).  It
// is issued from inline assembly on purpose: the compiler's automatic wait
// insertion cannot tell the ring slots apart and would wait for ALL outstanding
// loads before every LDS read; the waits for these loads are placed by hand
// (FLY_WAIT_VMCNT).  Unknown to the compiler's counters, they can only make its
// own vmcnt waits longer than needed, never shorter (register loads complete in
// order among themselves, and so do LDS-direct loads).  Between the two kinds
// there is NO order on this chip: a hand-counted wait is valid only while no
// register load of the wave is in flight (measured: a kernel that mixed them
// read LDS stages that had not landed).
// (M0 is reserved by the compiler, which warns about the clobber; nothing else
// in this file uses M0, and the clobber makes the compiler reload it if it did.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void global_to_lds16(const void* gptr, const void* lds_base) {
  const uint32_t lds_addr =
      (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)lds_base;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_addr), "v"(gptr)
               : "memory", "m0");
}
#pragma clang diagnostic pop
#define FLY_GLOBAL_TO_LDS16(gptr, lptr) global_to_lds16((const void*)(gptr), (const void*)(lptr))

// s_waitcnt vmcnt(n) only (expcnt and lgkmcnt left at "no wait").
#define FLY_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)
#define FLY_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(0xC07F)
// Workgroup barrier without the fence of __syncthreads (that fence would wait
// for ALL outstanding LDS-direct loads, also those of the stages still being
// prefetched).  The waits are placed by hand; the empty asm statements and the
// scheduling barriers keep the compiler from moving LDS accesses across it.
#define FLY_BARE_BARRIER()              \
  asm volatile("" ::: "memory");        \
  __builtin_amdgcn_sched_barrier(0);    \
  __builtin_amdgcn_s_barrier();         \
  __builtin_amdgcn_sched_barrier(0);    \
  asm volatile("" ::: "memory")

// ---- host-side launchers (defined in the kernel sources) -------------------
struct GemmPlan {
  int mt;      // 16-row tiles of activations held per workgroup (1,2,3,5,9)
  int nt;      // 16-column weight tiles per wave (1,2,4)
  int splits;  // split-K factor (partial results go to the workspace)
  int mblocks; // row blocks (activations beyond 144 rows re-stream the weights)
  int tiled;   // 0: weight-streaming kernel (mt, nt as above); else the LDS-tiled kernel with
               // workgroups of 256 columns x 128 (2), 192 (3), 256 (4) or 384 (6) rows (mt, nt unused)
  int wide;    // 0, or the weight-streaming kernel for 129..256 rows with this many 32-row tiles
               // (5, 6, 8); takes precedence over the other fields except splits
};

enum GemmEpilogue { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_LMHEAD = 2, EPI_LMSAMPLE = 3 };

hipError_t launch_pack_weight(const void* src, int64_t k_in, int64_t n_src, int dtype, void* dst,
                              int64_t n_dst, int64_t tile_offset, int64_t tile_stride,
                              hipStream_t st);

// bf16 weight-streaming GEMM: out = X[M,Kd] * W[Kd,N] (W packed).
//   EPI_PARTIAL: out = float partial[splits][M][N]
//   EPI_SWIGLU : out = bf16 a[M][N/2], a = silu(gate)*up (splits must be 1)
//   EPI_LMHEAD : out = RowStat-like float4 partial[M][nparts] (splits must be 1),
//                logits multiplied by row_scale[m] first
//   EPI_LMSAMPLE: EPI_LMHEAD, and smp.pick[M][nparts] receives the largest Gumbel-perturbed
//                logit of each part and its column
hipError_t launch_gemm_bf16(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale,
                            int M, int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st,
                            const LmSample& smp = LmSample{});
int gemm_bf16_lmhead_parts(int N, const GemmPlan& plan);
// LDS-tiled variant for large M (called through launch_gemm_bf16 when plan.tiled != 0).
hipError_t launch_gemm_bf16_tiled(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale,
                                  int M, int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st,
                                  const LmSample& smp = LmSample{});
int gemm_bf16_tiled_lmhead_parts(int N, int tiled);
// Weight-streaming variant for 129..256 rows (called through launch_gemm_bf16 when plan.wide != 0).
hipError_t launch_gemm_bf16_wide(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale, int M,
                                 int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st,
                                 const LmSample& smp = LmSample{});
int gemm_bf16_wide_lmhead_parts(int N);
int gemm_bf16_wide_cols();  // columns one workgroup covers
int gemm_bf16_tiled_rows(int tiled);
int gemm_bf16_tiled_cols(int tiled);

// fp32 GEMM (weights row-major [Kd,N]) with the same epilogues; no split-K.
hipError_t launch_gemm_f32(const float* X, const float* W, void* out, const float* row_scale, int M,
                           int N, int Kd, int epi, hipStream_t st, const LmSample& smp = LmSample{});
int gemm_f32_lmhead_parts(int N);

hipError_t launch_embed(const int32_t* tokens, const void* embed, int dtype, float* x, int M, int d,
                        int vocab, hipStream_t st);
// x[m] += sum_s partial[s][m] (partial may be NULL with splits = 0), then
// xn[m] = rmsnorm(x[m]) * gain in the activation dtype (xn may be NULL).
hipError_t launch_reduce_residual_norm(float* x, const float* partial, int splits, const void* gain,
                                       void* xn, int dtype, int M, int d, float eps, hipStream_t st);
hipError_t launch_rope_table(const int32_t* kv_len, float* table, int B, int K, int hd, float theta,
                             hipStream_t st);
// Sum split-K partials of the fused q/k/v projection, rotate q and k, write q
// (activation dtype) and append k, v to the cache.
hipError_t launch_qkv_epilogue(const float* partial, int splits, const float* rope, void* q,
                               void* kcache, void* vcache, const int32_t* kv_len, int dtype, int B,
                               int K, int Hq, int Hkv, int hd, int capacity, hipStream_t st);
// pick / sampled: the per-part picks of EPI_LMSAMPLE and the drawn token per row, or both NULL.
hipError_t launch_lmhead_combine(const float* partial, int nparts, int M, int V, int32_t* argmax,
                                 float* p_top1, float* h_norm, float* lse, hipStream_t st,
                                 const float* pick = nullptr, int32_t* sampled = nullptr);
hipError_t launch_accept(const int32_t* draft, int draft_stride, const int32_t* tgt,
                         const float* h_norm, const int32_t* kv_len, int B, int K, float theta,
                         int W, int32_t* accept_len, int32_t* next_token, int32_t* n_loose,
                         int32_t* kv_len_out, hipStream_t st);

struct AttnPlan {
  int nsplit;      // KV splits per (sequence, kv head)
  int chunk_keys;  // keys per split (multiple of 64)
  int qblocks;     // query-row blocks per (split, sequence, KV head): beyond 256 rows the
                   // rows are divided over several workgroups that stream the same keys
  int block_tiles; // 32-row tiles per query block (1..8)
};
extern std::atomic<int> g_attn_force_splits, g_attn_force_block_tiles;
extern std::atomic<int> g_wide_phase, g_tiled_phase, g_attn_phase;
AttnPlan plan_attention(int B, int K, int Hq, int Hkv, int max_total_len);
size_t attention_workspace_floats(int B, int K, int Hq, int Hkv, int hd, const AttnPlan& p);
hipError_t launch_attention_bf16(const bf16_t* q, const bf16_t* kcache, const bf16_t* vcache,
                                 const int32_t* kv_len, bf16_t* o, float* ws, int B, int K, int Hq,
                                 int Hkv, int hd, int capacity, const AttnPlan& p, hipStream_t st);
hipError_t launch_attention_f32(const float* q, const float* kcache, const float* vcache,
                                const int32_t* kv_len, float* o, int B, int K, int Hq, int Hkv,
                                int hd, int capacity, hipStream_t st);

// Decode loop (prompt-lookup drafter, end-of-round bookkeeping).
hipError_t launch_pld_draft(const int32_t* ctx, const int32_t* ctx_len, int ctx_capacity, int B, int K,
                            int n_max, int32_t* tokens, int32_t* ngram, hipStream_t st);
hipError_t launch_draft_prepare(const int32_t* ctx, const int32_t* ctx_len, int ctx_capacity, int B, int K,
                                int32_t* tok2, int32_t* len_steps, hipStream_t st);
hipError_t launch_draft_pick(const int32_t* argmax2, int B, int32_t* first, hipStream_t st);
hipError_t launch_draft_assemble(const int32_t* tok2, const int32_t* drafts, int B, int K, int32_t* tokens,
                                 hipStream_t st);
hipError_t launch_roll_forward(int32_t* ctx, int32_t* ctx_len, int32_t* kv_len, int ctx_capacity, int B,
                               int K, const int32_t* tokens, const int32_t* accept_len,
                               const int32_t* next_token, const int32_t* kv_len_out,
                               const int32_t* n_loose, int64_t* accepted_total, int32_t* rounds_done,
                               int64_t* loose_total, int32_t* trace_row, hipStream_t st);
