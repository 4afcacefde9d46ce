// (K+1)-query causal grouped-query attention against the KV cache
// (the attention inside the target's single verification pass; paper Sec. 2.1).
//
// For one (sequence, KV head) the G = Hq/Hkv query heads and the K+1 new
// positions give R = G*(K+1) query rows that all read the same keys and
// values, so the cache is streamed once per KV head and the work per key is a
// small dense contraction: matrix cores, with the cache as the streamed
// operand.  The cache axis is split over workgroups; each split produces an
// unnormalised output, a running maximum and a sum per query row, and a
// second kernel merges the splits.
//
// Layouts: keys [B, Hkv, capacity, hd]; values transposed [B, Hkv, hd, capacity];
// q and o [M, Hq*hd].  Query row r of a KV head is (position i = r / G,
// head kvh*G + r % G).
#include "fly_common.h"

#define ATT_HD 128
#define ATT_MAX_SPLITS 256
#define ATT_KC 64                      // keys per LDS stage
#define ATT_KROW (ATT_HD * 2)           // bytes per key row in LDS
#define ATT_VROW (ATT_KC * 2)           // bytes per V^T row in LDS
#define ATT_STAGE_BYTES (ATT_KC * ATT_KROW + ATT_HD * ATT_VROW)  // 32 KiB; two stages = 64 KiB
// Rows are stored unpadded; the 16-byte pieces of a row are permuted so that
// both the row-wise stores and the operand-order loads spread over all banks:
// key rows XOR the piece index with (key & 15), V^T rows with ((row >> 1) & 7).
#define ATT_KSWZ(key, piece) (((piece) ^ ((key) & 15)) * 16)
#define ATT_VSWZ(row, piece) (((piece) ^ (((row) >> 1) & 7)) * 16)

int g_attn_force_splits = 0;  // tuning knobs (0 = automatic)
int g_attn_force_qtw = 0;

AttnPlan plan_attention(int B, int K, int Hq, int Hkv, int max_total_len) {
  AttnPlan p;
  int G = Hq / Hkv;
  int R = G * (K + 1);
  int qt = (R + 15) / 16;
  p.qtw = qt <= 8 ? 1 : (qt <= 16 ? 2 : 3);  // up to eight waves per workgroup
  if (g_attn_force_qtw) p.qtw = g_attn_force_qtw;
  p.nwaves = (qt + p.qtw - 1) / p.qtw;  // caller guarantees <= 8
  int pairs = B * Hkv;
  int chunks = (max_total_len + ATT_KC - 1) / ATT_KC;
  if (chunks < 1) chunks = 1;
  // one workgroup per compute unit (the kernel's registers allow no more), at
  // least two stages per split
  int want = g_attn_force_splits ? g_attn_force_splits : (256 + pairs - 1) / pairs;
  int maxsplit = (chunks + 1) / 2;
  if (maxsplit < 1) maxsplit = 1;
  int ns = want < maxsplit ? want : maxsplit;
  if (ns > ATT_MAX_SPLITS) ns = ATT_MAX_SPLITS;
  if (ns < 1) ns = 1;
  int cps = (chunks + ns - 1) / ns;
  p.chunk_keys = cps * ATT_KC;
  p.nsplit = (chunks + cps - 1) / cps;
  return p;
}

size_t attention_workspace_floats(int B, int K, int Hq, int Hkv, int hd, const AttnPlan& p) {
  int G = Hq / Hkv;
  size_t R = (size_t)G * (K + 1);
  // per (pair, split): O [R, hd] + m [R] + l [R]
  return (size_t)B * Hkv * p.nsplit * R * (hd + 2);
}

template <int QTW, int NW>
__global__ __launch_bounds__(NW * 64) void attention_bf16_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kcache, const bf16_t* __restrict__ vcache,
    const int32_t* __restrict__ kv_len, float* __restrict__ ws, int K, int Hq, int Hkv, int capacity,
    int chunk_keys, float scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages
  constexpr int nthreads = NW * 64;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: scalar branches
  const int g = lane >> 4, c16 = lane & 15;
  const int split = blockIdx.x, pair = blockIdx.y, nsplit = gridDim.x;
  const int b = pair / Hkv, kvh = pair % Hkv;
  const int G = Hq / Hkv;
  const int R = G * (K + 1);
  const int L = kv_len[b];
  int total = L + K + 1;  // keys visible to the last query
  if (total > capacity) total = capacity;  // the host checks this bound; never read past the slab
  const int key_begin = split * chunk_keys;
  int key_end = key_begin + chunk_keys;
  if (key_end > total) key_end = total;

  const bf16_t* kbase = kcache + ((int64_t)b * Hkv + kvh) * (int64_t)capacity * ATT_HD;
  const bf16_t* vbase = vcache + ((int64_t)b * Hkv + kvh) * (int64_t)ATT_HD * capacity;

  // ---- this wave's query tiles: operand B of S^T = K Q^T, lane holds
  // Q[row = 16*tile + c16][hd = 32*kk + 8g .. +8]
  u32x4 qf[QTW][4];
  int qrow[QTW];   // query row of this lane's column, or -1
  int qlimit[QTW]; // number of visible keys for that row
#pragma unroll
  for (int t = 0; t < QTW; ++t) {
    int r = (wave * QTW + t) * 16 + c16;
    bool ok = r < R;
    qrow[t] = ok ? r : -1;
    int rc = ok ? r : R - 1;  // clamp: the load is unconditional, the value is masked
    int i = rc / G, gq = rc % G;
    qlimit[t] = ok ? L + i + 1 : 0;
    const bf16_t* qp = q + ((int64_t)(b * (K + 1) + i) * Hq + kvh * G + gq) * ATT_HD;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4 v = *(const u32x4*)(qp + 32 * kk + 8 * g);
      qf[t][kk] = ok ? v : u32x4{0u, 0u, 0u, 0u};
    }
  }

  f32x4 oacc[QTW][8];  // O^T[hd = 16*ht + 4g + r][row c16]
  float mrun[QTW], lrun[QTW];
#pragma unroll
  for (int t = 0; t < QTW; ++t) {
    mrun[t] = -INFINITY;
    lrun[t] = 0.f;
#pragma unroll
    for (int ht = 0; ht < 8; ++ht) oacc[t][ht] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // ---- cooperative stage load: K part 64 keys x 256 B, V^T part 128 rows x 128 B,
  // 16 bytes per thread per item; items [0, 1024) are K, [1024, 2048) are V.
  constexpr int ITEMS = (ATT_KC * ATT_HD * 2 * 2) / 16;  // 2048
  constexpr int MAX_PER_THREAD = ITEMS / nthreads;       // 8 (four waves) or 4 (eight waves)
  u32x4 stgA[MAX_PER_THREAD], stgB[MAX_PER_THREAD];  // two stages in flight

  // Loads are unconditional and branch-free so that all of a stage's loads are
  // in flight together: a stage starts at a multiple of 64 below key_end and the
  // capacity is a multiple of 64, so rows kstart..kstart+63 exist in the slab.
  // Rows / columns at or past key_end hold whatever the allocation held
  // (possibly NaN patterns; 0 * NaN would poison the sums): they are zeroed
  // when the stage is written to LDS, which only the last stage needs.
  auto load_stage = [&](u32x4 (&stg)[MAX_PER_THREAD], int kstart) {
#pragma unroll
    for (int it = 0; it < MAX_PER_THREAD; ++it) {
      const int item = it * nthreads + tid;
      if (it < MAX_PER_THREAD / 2) {  // K half (compile-time split)
        int key = item >> 4, piece = item & 15;
        stg[it] = *(const u32x4*)(kbase + (int64_t)(kstart + key) * ATT_HD + piece * 8);
      } else {
        int it2 = item - ITEMS / 2;
        int row = it2 >> 3, piece = it2 & 7;
        stg[it] = *(const u32x4*)(vbase + (int64_t)row * capacity + kstart + piece * 8);
      }
    }
  };
  auto store_stage = [&](const u32x4 (&stg)[MAX_PER_THREAD], int stage, int kstart) {
    unsigned char* base = smem + stage * ATT_STAGE_BYTES;
    const bool tail = kstart + ATT_KC > key_end;  // workgroup-uniform
#pragma unroll
    for (int it = 0; it < MAX_PER_THREAD; ++it) {
      const int item = it * nthreads + tid;
      u32x4 v = stg[it];
      if (it < MAX_PER_THREAD / 2) {
        int key = item >> 4, piece = item & 15;
        if (tail && kstart + key >= key_end) v = u32x4{0u, 0u, 0u, 0u};
        *(u32x4*)(base + key * ATT_KROW + ATT_KSWZ(key, piece)) = v;
      } else {
        int it2 = item - ITEMS / 2;
        int row = it2 >> 3, piece = it2 & 7;
        if (tail) {
          int nvalid = key_end - (kstart + piece * 8);  // valid keys in this 8-key piece
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            uint32_t keep = (2 * w < nvalid ? 0xFFFFu : 0u) | (2 * w + 1 < nvalid ? 0xFFFF0000u : 0u);
            v[w] &= keep;
          }
        }
        *(u32x4*)(base + ATT_KC * ATT_KROW + row * ATT_VROW + ATT_VSWZ(row, piece)) = v;
      }
    }
  };

  const int nstages = key_end > key_begin ? (key_end - key_begin + ATT_KC - 1) / ATT_KC : 0;

  // One 64-key stage from LDS buffer `stage`, whose first key is kstart.
  //
  // Probabilities are formed relative to an INTEGER base-2 exponent n >= max s',
  // s' = (q.k) * log2(e)/sqrt(hd), n = ceil of the running maximum: when the
  // maximum grows, earlier terms are rescaled by an exact power of two, which
  // commutes with the bf16 rounding of P.  The result is the same as rounding
  // 2^(s' - n_final) once, independent of how the cache is chunked or split.
  //
  // The per-score vector work is what bounds this kernel once the loads are
  // hidden, so it is kept minimal: the causal / tail mask is applied only in
  // stages that reach past the prefix (uniform branch), the scale is folded
  // into one fused multiply-add with the exponent, and the accumulators are
  // rescaled only when some row's exponent actually changed.
  const bool wave_has_rows = wave * QTW * 16 < R;
  auto compute_stage = [&](int stage, int kstart) {
    if (!wave_has_rows) return;  // this wave only helps with the loads
    const unsigned char* kb = smem + stage * ATT_STAGE_BYTES;
    const unsigned char* vb = kb + ATT_KC * ATT_KROW;

    // S^T = K Q^T: 4 key tiles of 16; lane holds S[key = 16*kt + 4g + r][row c16].
    // Each key fragment is read from LDS once and used for all of the wave's query tiles.
    f32x4 sacc[QTW][4];
#pragma unroll
    for (int t = 0; t < QTW; ++t)
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) sacc[t][kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        u32x4 araw = *(const u32x4*)(kb + (kt * 16 + c16) * ATT_KROW + ATT_KSWZ(c16, 4 * kk + g));
        bf16x8 a = __builtin_bit_cast(bf16x8, araw);
#pragma unroll
        for (int t = 0; t < QTW; ++t)
          sacc[t][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, qf[t][kk]),
                                                                sacc[t][kt], 0, 0, 0);
      }
    }

    const bool need_mask = kstart + ATT_KC > L + 1;  // keys below L+1 are visible to every row
    uint32_t pb[QTW][4][2];  // bf16 pairs: P[key 16*kt + 4g + {0,1}], {2,3}
#pragma unroll
    for (int t = 0; t < QTW; ++t) {
      if (need_mask) {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            int key = kstart + kt * 16 + 4 * g + r;
            if (key >= qlimit[t]) sacc[t][kt][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
        mx = fmaxf(mx, fmaxf(fmaxf(sacc[t][kt][0], sacc[t][kt][1]), fmaxf(sacc[t][kt][2], sacc[t][kt][3])));
      mx = fmaxf(mx, __shfl_xor(mx, 16, FLY_WAVE));
      mx = fmaxf(mx, __shfl_xor(mx, 32, FLY_WAVE));
      const float mnew = fmaxf(mrun[t], ceilf(mx * scale));  // scale > 0: max commutes with it
      // rows with nothing visible yet keep n = -inf; avoid inf - inf
      const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
      if (__ballot(mnew != mrun[t]) != 0ull) {  // wave-uniform: some row's exponent grew
        const float corr = fast_exp2(mrun[t] - msafe);  // exact power of two (0 when mrun = -inf)
        lrun[t] *= corr;
#pragma unroll
        for (int ht = 0; ht < 8; ++ht) oacc[t][ht] *= corr;
        mrun[t] = mnew;
      }
      float lsum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) {
        float p0 = fast_exp2(fmaf(sacc[t][kt][0], scale, -msafe));
        float p1 = fast_exp2(fmaf(sacc[t][kt][1], scale, -msafe));
        float p2 = fast_exp2(fmaf(sacc[t][kt][2], scale, -msafe));
        float p3 = fast_exp2(fmaf(sacc[t][kt][3], scale, -msafe));
        lsum += (p0 + p1) + (p2 + p3);
        pb[t][kt][0] = pack_bf2_hw(p0, p1);
        pb[t][kt][1] = pack_bf2_hw(p2, p3);
      }
      lrun[t] += lsum;
    }

    // O^T += V^T P^T.  k-step ks covers keys 32ks..32ks+31 with the operand
    // index order (4g..4g+3 of tile 2ks, then 4g..4g+3 of tile 2ks+1); each V^T
    // fragment is read once and used for all query tiles.
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      bf16x8 bop[QTW];
#pragma unroll
      for (int t = 0; t < QTW; ++t) {
        u32x4 braw;
        braw.x = pb[t][2 * ks][0];
        braw.y = pb[t][2 * ks][1];
        braw.z = pb[t][2 * ks + 1][0];
        braw.w = pb[t][2 * ks + 1][1];
        bop[t] = __builtin_bit_cast(bf16x8, braw);
      }
#pragma unroll
      for (int ht = 0; ht < 8; ++ht) {
        // keys 32ks + 4g .. +3 sit in piece 4ks + g/2 at byte 8(g&1); keys +16 two pieces on
        const int vrow = ht * 16 + c16;
        const unsigned char* vr = vb + vrow * ATT_VROW + 8 * (g & 1);
        u32x2 lo = *(const u32x2*)(vr + ATT_VSWZ(vrow, 4 * ks + (g >> 1)));
        u32x2 hi = *(const u32x2*)(vr + ATT_VSWZ(vrow, 4 * ks + (g >> 1) + 2));
        u32x4 araw;
        araw.x = lo.x;
        araw.y = lo.y;
        araw.z = hi.x;
        araw.w = hi.y;
        bf16x8 a = __builtin_bit_cast(bf16x8, araw);
#pragma unroll
        for (int t = 0; t < QTW; ++t)
          oacc[t][ht] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bop[t], oacc[t][ht], 0, 0, 0);
      }
    }
  };

  // Pipeline: while stage i is multiplied out of LDS, stage i+1 sits in
  // registers waiting to be written to the other LDS buffer and stage i+2 is
  // being loaded.  Register sets alternate (A, B), LDS buffers alternate (0, 1).
  // The steady-state loop has no conditionals so that the waits before the LDS
  // writes cover only the older of the two register sets.
#define KST(i) (key_begin + (i) * ATT_KC)
  if (nstages > 0) load_stage(stgA, KST(0));
  if (nstages > 1) load_stage(stgB, KST(1));
  if (nstages > 0) store_stage(stgA, 0, KST(0));
  __syncthreads();
  int sidx = 0;
  while (sidx + 3 < nstages) {
    load_stage(stgA, KST(sidx + 2));
    compute_stage(0, KST(sidx));
    store_stage(stgB, 1, KST(sidx + 1));
    __syncthreads();
    load_stage(stgB, KST(sidx + 3));
    compute_stage(1, KST(sidx + 1));
    store_stage(stgA, 0, KST(sidx + 2));
    __syncthreads();
    sidx += 2;
  }
  for (; sidx < nstages; sidx += 2) {  // tail: at most three stages, with checks
    if (sidx + 2 < nstages) load_stage(stgA, KST(sidx + 2));
    compute_stage(0, KST(sidx));
    if (sidx + 1 < nstages) store_stage(stgB, 1, KST(sidx + 1));
    __syncthreads();
    if (sidx + 1 >= nstages) break;
    if (sidx + 3 < nstages) load_stage(stgB, KST(sidx + 3));
    compute_stage(1, KST(sidx + 1));
    if (sidx + 2 < nstages) store_stage(stgA, 0, KST(sidx + 2));
    __syncthreads();
  }
#undef KST

  // ---- write this split's partial: O [R, hd], m [R], l [R]
  float* obase = ws + ((int64_t)pair * nsplit + split) * (int64_t)R * (ATT_HD + 2);
  float* mbase = obase + (int64_t)R * ATT_HD;
  float* lbase = mbase + R;
#pragma unroll
  for (int t = 0; t < QTW; ++t) {
    float l = lrun[t];
    l += __shfl_xor(l, 16, FLY_WAVE);
    l += __shfl_xor(l, 32, FLY_WAVE);
    int r = qrow[t];
    if (r >= 0) {
#pragma unroll
      for (int ht = 0; ht < 8; ++ht)
        *(f32x4*)(obase + (int64_t)r * ATT_HD + ht * 16 + 4 * g) = oacc[t][ht];
      if (g == 0) {
        mbase[r] = mrun[t];
        lbase[r] = l;
      }
    }
  }
}

// Merge the splits: o = sum_s O_s 2^(n_s - n) / sum_s l_s 2^(n_s - n), n = max_s n_s.
// grid (R, B*Hkv), block 128 (one thread per head-dim element).
__global__ __launch_bounds__(ATT_HD) void attention_combine_kernel(const float* __restrict__ ws,
                                                                   bf16_t* __restrict__ o, int K,
                                                                   int Hq, int Hkv, int nsplit) {
  __shared__ float wgt[ATT_MAX_SPLITS];  // 2^(n_s - n) per split, 0 for empty splits
  __shared__ float lw[ATT_MAX_SPLITS];   // l_s * weight
  const int r = blockIdx.x, pair = blockIdx.y, e = threadIdx.x;
  const int b = pair / Hkv, kvh = pair % Hkv;
  const int G = Hq / Hkv, R = G * (K + 1);
  const float* base = ws + (int64_t)pair * nsplit * (int64_t)R * (ATT_HD + 2);
  const int64_t sstride = (int64_t)R * (ATT_HD + 2);
  // every thread finds the largest exponent (the loads are the same for all
  // threads and independent of each other)
  float mx = -INFINITY;
  for (int s = 0; s < nsplit; ++s) mx = fmaxf(mx, base[s * sstride + (int64_t)R * ATT_HD + r]);
  for (int s = e; s < nsplit; s += ATT_HD) {
    const float* sb = base + s * sstride + (int64_t)R * ATT_HD;
    float ms = sb[r], ls = sb[R + r];
    float w = ls > 0.f ? fast_exp2(ms - mx) : 0.f;  // integer exponents: an exact power of two
    wgt[s] = w;
    lw[s] = ls * w;
  }
  __syncthreads();
  float num = 0.f, den = 0.f;
  // split order is fixed, so the sum does not depend on scheduling
#pragma unroll 4
  for (int s = 0; s < nsplit; ++s) {
    num = fmaf(base[s * sstride + (int64_t)r * ATT_HD + e], wgt[s], num);
    den += lw[s];
  }
  const int i = r / G, gq = r % G;
  o[((int64_t)(b * (K + 1) + i) * Hq + kvh * G + gq) * ATT_HD + e] = f2bf(num / den);
}

hipError_t launch_attention_bf16(const bf16_t* q, const bf16_t* kcache, const bf16_t* vcache,
                                 const int32_t* kv_len, bf16_t* o, float* ws, int B, int K, int Hq,
                                 int Hkv, int hd, int capacity, const AttnPlan& p, hipStream_t st) {
  // Shapes the kernel assumes.
  if (hd != ATT_HD || Hq % Hkv != 0 || capacity % 64 != 0 || p.chunk_keys % ATT_KC != 0)
    return hipErrorInvalidValue;
  if (p.nwaves < 1 || p.nwaves > 8 || p.qtw < 1 || p.qtw > 3) return hipErrorInvalidValue;
  if (p.nsplit < 1 || p.nsplit > ATT_MAX_SPLITS) return hipErrorInvalidValue;
  int G = Hq / Hkv, R = G * (K + 1);
  if (p.nwaves * p.qtw * 16 < R) return hipErrorInvalidValue;
  // the stage loader gives each thread 2048 / nthreads items: 4 or 8 waves
  int nw = p.nwaves <= 4 ? 4 : 8;
  dim3 grid(p.nsplit, B * Hkv), block(nw * 64);
  size_t smem = 2 * ATT_STAGE_BYTES;
  float scale = (float)(1.4426950408889634 / sqrt((double)hd));  // log2(e) / sqrt(hd)
#define FLY_ATT_LAUNCH(QTW_, NW_)                                                                   \
  hipLaunchKernelGGL((attention_bf16_kernel<QTW_, NW_>), grid, block, smem, st, q, kcache, vcache,   \
                     kv_len, ws, K, Hq, Hkv, capacity, p.chunk_keys, scale)
  if (nw == 4) {
    if (p.qtw == 1) FLY_ATT_LAUNCH(1, 4);
    else if (p.qtw == 2) FLY_ATT_LAUNCH(2, 4);
    else FLY_ATT_LAUNCH(3, 4);
  } else {
    if (p.qtw == 1) FLY_ATT_LAUNCH(1, 8);
    else if (p.qtw == 2) FLY_ATT_LAUNCH(2, 8);
    else FLY_ATT_LAUNCH(3, 8);
  }
#undef FLY_ATT_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attention_combine_kernel, dim3(R, B * Hkv), dim3(ATT_HD), 0, st, ws, o, K, Hq, Hkv,
                     p.nsplit);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// fp32 attention (tiny configuration): one wavefront per (row m, query head).
// Lanes own keys for the scores and head-dim elements for the output.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void attention_f32_kernel(const float* __restrict__ q,
                                                           const float* __restrict__ kcache,
                                                           const float* __restrict__ vcache,
                                                           const int32_t* __restrict__ kv_len,
                                                           float* __restrict__ o, int K, int Hq,
                                                           int Hkv, int hd, int capacity, float scale) {
  __shared__ float qs[128];
  const int m = blockIdx.x, a = blockIdx.y, lane = threadIdx.x;
  const int b = m / (K + 1), i = m % (K + 1);
  const int G = Hq / Hkv, kvh = a / G;
  const int nvis = kv_len[b] + i + 1;
  const float* qp = q + ((int64_t)m * Hq + a) * hd;
  for (int e = lane; e < hd; e += 64) qs[e] = qp[e];
  __syncthreads();
  const float* kb = kcache + ((int64_t)b * Hkv + kvh) * (int64_t)capacity * hd;
  const float* vb = vcache + ((int64_t)b * Hkv + kvh) * (int64_t)hd * capacity;
  float mrun = -INFINITY, lrun = 0.f, acc0 = 0.f, acc1 = 0.f;  // lane owns elements lane, lane+64
  for (int k0 = 0; k0 < nvis; k0 += 64) {
    int key = k0 + lane;
    float s = -INFINITY;
    if (key < nvis) {
      const float* kr = kb + (int64_t)key * hd;
      float dot = 0.f;
      for (int e = 0; e < hd; ++e) dot = fmaf(qs[e], kr[e], dot);
      s = dot * scale;
    }
    float mnew = fmaxf(mrun, wave_max(s));
    float corr = __expf(mrun - mnew);
    float p = (key < nvis) ? __expf(s - mnew) : 0.f;
    lrun = lrun * corr + wave_sum(p);
    acc0 *= corr;
    acc1 *= corr;
    int cnt = min(64, nvis - k0);
    for (int jj = 0; jj < cnt; ++jj) {
      float pj = __shfl(p, jj, FLY_WAVE);
      if (lane < hd) acc0 = fmaf(pj, vb[(int64_t)lane * capacity + k0 + jj], acc0);
      if (lane + 64 < hd) acc1 = fmaf(pj, vb[(int64_t)(lane + 64) * capacity + k0 + jj], acc1);
    }
    mrun = mnew;
  }
  float* op = o + ((int64_t)m * Hq + a) * hd;
  if (lane < hd) op[lane] = acc0 / lrun;
  if (lane + 64 < hd) op[lane + 64] = acc1 / lrun;
}

hipError_t launch_attention_f32(const float* q, const float* kcache, const float* vcache,
                                const int32_t* kv_len, float* o, int B, int K, int Hq, int Hkv,
                                int hd, int capacity, hipStream_t st) {
  if (hd > 128 || hd < 1 || Hq % Hkv != 0) return hipErrorInvalidValue;
  float scale = 1.0f / sqrtf((float)hd);
  hipLaunchKernelGGL(attention_f32_kernel, dim3(B * (K + 1), Hq), dim3(64), 0, st, q, kcache, vcache,
                     kv_len, o, K, Hq, Hkv, hd, capacity, scale);
  return hipGetLastError();
}
