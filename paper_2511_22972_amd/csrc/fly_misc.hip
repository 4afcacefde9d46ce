// Small kernels around the GEMMs: embedding gather, residual + RMSNorm,
// rotary tables, the q/k/v epilogue that appends to the KV cache, the
// combine step of the fused LM-head statistics (Eq. 1, Eq. 5) and FLy's
// acceptance rule (Eqs. 2-11; Algorithm 1 steps 3-4).
#include "fly_common.h"

// ---------------------------------------------------------------------------
// x[m] = E[tok[m]]  (fp32 residual stream)
// ---------------------------------------------------------------------------
template <typename WT>
__global__ void embed_kernel(const int32_t* __restrict__ tokens, const WT* __restrict__ embed,
                             float* __restrict__ x, int d, int vocab) {
  int m = blockIdx.x;
  int tok = tokens[m];
  // token ids outside the vocabulary would read out of bounds: clamp
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
  const WT* e = embed + (int64_t)tok * d;
  float* xr = x + (int64_t)m * d;
  if constexpr (sizeof(WT) == 2) {
    // rows are multiples of 32 elements and 16-byte aligned: eight bf16 per load
    for (int i = threadIdx.x * 8; i < d; i += blockDim.x * 8) {
      const u32x4 v = *(const u32x4*)(e + i);
      *(f32x4*)(xr + i) = f32x4{__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u),
                                __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xFFFF0000u)};
      *(f32x4*)(xr + i + 4) = f32x4{__uint_as_float(v.z << 16), __uint_as_float(v.z & 0xFFFF0000u),
                                    __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xFFFF0000u)};
    }
  } else {
    for (int i = threadIdx.x; i < d; i += blockDim.x) xr[i] = Act<WT>::ld(e + i);
  }
}

hipError_t launch_embed(const int32_t* tokens, const void* embed, int dtype, float* x, int M, int d,
                        int vocab, hipStream_t st) {
  if (dtype == FLY_BF16)
    hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(M), dim3(256), 0, st, tokens, (const bf16_t*)embed, x, d, vocab);
  else
    hipLaunchKernelGGL(embed_kernel<float>, dim3(M), dim3(256), 0, st, tokens, (const float*)embed, x, d, vocab);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// x[m] += sum_s partial[s][m];  xn[m] = x[m] * rsqrt(mean(x[m]^2) + eps) * gain
// One workgroup per row.  The split-K partial sums are added in split order,
// so the result does not depend on scheduling.
// ---------------------------------------------------------------------------
#define RRN_THREADS 1024
template <typename AT>
__global__ __launch_bounds__(RRN_THREADS) void reduce_residual_norm_kernel(
    float* __restrict__ x, const float* __restrict__ partial, int splits, const AT* __restrict__ gain,
    AT* __restrict__ xn, int M, int d, float eps) {
  __shared__ float wsum[RRN_THREADS / 64];
  const int m = blockIdx.x;
  float* xr = x + (int64_t)m * d;
  // Only M rows exist, so the row is spread over 16 waves to keep enough loads
  // in flight.  A thread owns groups of four elements RRN_THREADS*4 apart; up to
  // RRN_KEEP of them stay in registers between the two passes.  The partials of
  // one group are fetched four splits at a time (independent loads, one wait)
  // and added in split order, so the sum does not depend on the batching.
  constexpr int RRN_KEEP = 4;
  f32x4 keep[RRN_KEEP];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < RRN_KEEP; ++it) keep[it] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto summed = [&](int i) {
    f32x4 v = *(f32x4*)(xr + i);
    const float* pp = partial + (int64_t)m * d + i;
    const int64_t sstride = (int64_t)M * d;
    int s = 0;
    for (; s + 4 <= splits; s += 4) {
      f32x4 p0 = *(const f32x4*)(pp + (s + 0) * sstride);
      f32x4 p1 = *(const f32x4*)(pp + (s + 1) * sstride);
      f32x4 p2 = *(const f32x4*)(pp + (s + 2) * sstride);
      f32x4 p3 = *(const f32x4*)(pp + (s + 3) * sstride);
      v += p0;
      v += p1;
      v += p2;
      v += p3;
    }
    for (; s < splits; ++s) v += *(const f32x4*)(pp + s * sstride);
    if (splits > 0) *(f32x4*)(xr + i) = v;
    return v;
  };
#pragma unroll
  for (int it = 0; it < RRN_KEEP; ++it) {
    const int i = (it * RRN_THREADS + threadIdx.x) * 4;
    if (i < d) {
      f32x4 v = summed(i);
      keep[it] = v;
      ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
  }
  for (int i = (RRN_KEEP * RRN_THREADS + threadIdx.x) * 4; i < d; i += RRN_THREADS * 4) {  // very wide rows
    f32x4 v = summed(i);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  if (xn == nullptr) return;
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < RRN_THREADS / 64; ++w) tot += wsum[w];
  float inv = 1.0f / sqrtf(tot / (float)d + eps);
  AT* o = xn + (int64_t)m * d;
  auto emit = [&](int i, const f32x4& v) {
    if constexpr (sizeof(AT) == 2) {
      const u32x2 gp = *(const u32x2*)(gain + i);  // four bf16 gains
      const float g0 = __uint_as_float(gp.x << 16), g1 = __uint_as_float(gp.x & 0xFFFF0000u);
      const float g2 = __uint_as_float(gp.y << 16), g3 = __uint_as_float(gp.y & 0xFFFF0000u);
      u32x2 pk;
      pk.x = pack_bf2(v.x * inv * g0, v.y * inv * g1);
      pk.y = pack_bf2(v.z * inv * g2, v.w * inv * g3);
      *(u32x2*)(o + i) = pk;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) Act<AT>::st(o + i + e, v[e] * inv * Act<AT>::ld(gain + i + e));
    }
  };
#pragma unroll
  for (int it = 0; it < RRN_KEEP; ++it) {
    const int i = (it * RRN_THREADS + threadIdx.x) * 4;
    if (i < d) emit(i, keep[it]);
  }
  for (int i = (RRN_KEEP * RRN_THREADS + threadIdx.x) * 4; i < d; i += RRN_THREADS * 4)
    emit(i, *(f32x4*)(xr + i));
}

hipError_t launch_reduce_residual_norm(float* x, const float* partial, int splits, const void* gain,
                                       void* xn, int dtype, int M, int d, float eps, hipStream_t st) {
  if (d % 4 != 0) return hipErrorInvalidValue;
  if (dtype == FLY_BF16)
    hipLaunchKernelGGL(reduce_residual_norm_kernel<bf16_t>, dim3(M), dim3(RRN_THREADS), 0, st, x, partial,
                       splits, (const bf16_t*)gain, (bf16_t*)xn, M, d, eps);
  else
    hipLaunchKernelGGL(reduce_residual_norm_kernel<float>, dim3(M), dim3(RRN_THREADS), 0, st, x, partial,
                       splits, (const float*)gain, (float*)xn, M, d, eps);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Rotary table: for row m = b*(K+1)+i at position kv_len[b]+i and frequency
// index f: (cos, sin)(pos * theta^(-2f/hd)).  Angles are formed in fp64 (a
// position of 3e4 times a frequency near 1 loses three digits in fp32) and the
// results stored as fp32.
// ---------------------------------------------------------------------------
__global__ void rope_table_kernel(const int32_t* __restrict__ kv_len, float* __restrict__ table, int B,
                                  int K, int hd, float theta) {
  int half = hd / 2;
  int gid = blockIdx.x * blockDim.x + threadIdx.x;
  int total = B * (K + 1) * half;
  if (gid >= total) return;
  int f = gid % half, m = gid / half;
  int b = m / (K + 1), i = m % (K + 1);
  double pos = (double)(kv_len[b] + i);
  double inv_freq = pow((double)theta, -2.0 * (double)f / (double)hd);
  double ang = pos * inv_freq;
  table[2 * (int64_t)gid] = (float)cos(ang);
  table[2 * (int64_t)gid + 1] = (float)sin(ang);
}

hipError_t launch_rope_table(const int32_t* kv_len, float* table, int B, int K, int hd, float theta,
                             hipStream_t st) {
  int total = B * (K + 1) * (hd / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((total + 127) / 128), dim3(128), 0, st, kv_len, table, B,
                     K, hd, theta);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// q/k/v epilogue: sum split-K partials of the fused projection
// [M, (Hq+2Hkv)*hd], rotate q and k heads (pairs (e, e+hd/2)), write q and
// append k (row-major) and v (transposed) to the cache at row kv_len[b]+i.
// grid (M, Hq+2Hkv), block hd/2.
// ---------------------------------------------------------------------------
template <typename AT>
__global__ void qkv_epilogue_kernel(const float* __restrict__ partial, int splits,
                                    const float* __restrict__ rope, AT* __restrict__ q,
                                    AT* __restrict__ kcache, AT* __restrict__ vcache,
                                    const int32_t* __restrict__ kv_len, int M, int K, int Hq, int Hkv,
                                    int hd, int capacity) {
  const int m = blockIdx.x, head = blockIdx.y, e = threadIdx.x, half = hd / 2;
  const int N = (Hq + 2 * Hkv) * hd;
  // split partials are fetched four at a time (independent loads, one wait) and
  // added in split order
  float lo = 0.f, hi = 0.f;
  const float* p = partial + (int64_t)m * N + head * hd + e;
  const int64_t sstride = (int64_t)M * N;
  int s = 0;
  for (; s + 4 <= splits; s += 4) {
    float a0 = p[(s + 0) * sstride], b0 = p[(s + 0) * sstride + half];
    float a1 = p[(s + 1) * sstride], b1 = p[(s + 1) * sstride + half];
    float a2 = p[(s + 2) * sstride], b2 = p[(s + 2) * sstride + half];
    float a3 = p[(s + 3) * sstride], b3 = p[(s + 3) * sstride + half];
    lo += a0; lo += a1; lo += a2; lo += a3;
    hi += b0; hi += b1; hi += b2; hi += b3;
  }
  for (; s < splits; ++s) {
    lo += p[s * sstride];
    hi += p[s * sstride + half];
  }
  const int b = m / (K + 1), i = m % (K + 1);
  if (head < Hq + Hkv) {
    float c = rope[2 * ((int64_t)m * half + e)], sn = rope[2 * ((int64_t)m * half + e) + 1];
    float rlo = lo * c - hi * sn, rhi = hi * c + lo * sn;
    lo = rlo;
    hi = rhi;
  }
  if (head < Hq) {
    AT* o = q + (int64_t)m * Hq * hd + head * hd;
    Act<AT>::st(o + e, lo);
    Act<AT>::st(o + e + half, hi);
    return;
  }
  const int pos = kv_len[b] + i;
  if (pos >= capacity) return;  // host checks the bound; never write outside the cache
  if (head < Hq + Hkv) {
    int kvh = head - Hq;
    AT* o = kcache + (((int64_t)b * Hkv + kvh) * capacity + pos) * hd;
    Act<AT>::st(o + e, lo);
    Act<AT>::st(o + e + half, hi);
  } else {
    int kvh = head - Hq - Hkv;
    AT* o = vcache + ((int64_t)b * Hkv + kvh) * hd * (int64_t)capacity + pos;
    Act<AT>::st(o + (int64_t)e * capacity, lo);
    Act<AT>::st(o + (int64_t)(e + half) * capacity, hi);
  }
}

hipError_t launch_qkv_epilogue(const float* partial, int splits, const float* rope, void* q,
                               void* kcache, void* vcache, const int32_t* kv_len, int dtype, int B,
                               int K, int Hq, int Hkv, int hd, int capacity, hipStream_t st) {
  int M = B * (K + 1);
  dim3 grid(M, Hq + 2 * Hkv), block(hd / 2);
  if (dtype == FLY_BF16)
    hipLaunchKernelGGL(qkv_epilogue_kernel<bf16_t>, grid, block, 0, st, partial, splits, rope,
                       (bf16_t*)q, (bf16_t*)kcache, (bf16_t*)vcache, kv_len, M, K, Hq, Hkv, hd, capacity);
  else
    hipLaunchKernelGGL(qkv_epilogue_kernel<float>, grid, block, 0, st, partial, splits, rope,
                       (float*)q, (float*)kcache, (float*)vcache, kv_len, M, K, Hq, Hkv, hd, capacity);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// LM-head combine: merge the per-wave statistics of one row over all column
// groups, then lse = m + ln s, H = ln s - t/s, h = H / ln V (Eq. 5),
// p_top1 = 1/s (the argmax logit is m), argmax = lowest maximal index (Eq. 1).
// With pick != NULL also the drawn token: the column of the largest
// Gumbel-perturbed logit over all parts (lowest column on ties).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lmhead_combine_kernel(const f32x4* __restrict__ partial,
                                                             int nparts, int V,
                                                             int32_t* __restrict__ argmax,
                                                             float* __restrict__ p_top1,
                                                             float* __restrict__ h_norm,
                                                             float* __restrict__ lse,
                                                             const float* __restrict__ pick,
                                                             int32_t* __restrict__ sampled) {
  __shared__ RowStat wst[4];
  __shared__ RowPick wpk[4];
  const int m = blockIdx.x;
  RowStat st = stat_empty();
  RowPick pk = pick_empty();
  for (int p = threadIdx.x; p < nparts; p += 256) {
    f32x4 w = partial[(int64_t)m * nparts + p];
    RowStat o{w.x, w.y, w.z, __float_as_int(w.w)};
    st = stat_merge(st, o);
    if (pick != nullptr) {
      const float* pp = pick + 2 * ((int64_t)m * nparts + p);
      pk = pick_merge(pk, RowPick{pp[0], __float_as_int(pp[1])});
    }
  }
  if (pick != nullptr) {  // uniform over the workgroup
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) pk = pick_merge(pk, pick_shfl_xor(pk, off));
    if ((threadIdx.x & 63) == 0) wpk[threadIdx.x >> 6] = pk;
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) st = stat_merge(st, stat_shfl_xor(st, off));
  if ((threadIdx.x & 63) == 0) wst[threadIdx.x >> 6] = st;
  __syncthreads();
  if (threadIdx.x == 0) {
    RowStat r = stat_merge(stat_merge(wst[0], wst[1]), stat_merge(wst[2], wst[3]));
    float ln_s = logf(r.s);
    float H = ln_s - r.t / r.s;
    argmax[m] = r.idx;
    p_top1[m] = 1.0f / r.s;
    h_norm[m] = H / logf((float)V);
    if (lse != nullptr) lse[m] = r.m + ln_s;
    if (pick != nullptr) {
      RowPick q = pick_merge(pick_merge(wpk[0], wpk[1]), pick_merge(wpk[2], wpk[3]));
      // a row whose logits are all -inf has no perturbed maximum: fall back to the argmax
      sampled[m] = q.idx != 0x7fffffff ? q.idx : r.idx;
    }
  }
}

hipError_t launch_lmhead_combine(const float* partial, int nparts, int M, int V, int32_t* argmax,
                                 float* p_top1, float* h_norm, float* lse, hipStream_t st,
                                 const float* pick, int32_t* sampled) {
  if ((pick == nullptr) != (sampled == nullptr)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(lmhead_combine_kernel, dim3(M), dim3(256), 0, st, (const f32x4*)partial, nparts,
                     V, argmax, p_top1, h_norm, lse, pick, sampled);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Acceptance rule: one wavefront per sequence, lane l <-> draft position
// j = l+1 (K <= 63).  A mismatch at j is rejected when h_j < theta (strict
// gate, Eq. 6), when the window does not fit (j + W > K, Sec. 2.2 boundary
// rule) or when one of positions j+1..j+W mismatches (Eqs. 8-9).  s is the
// first rejected position or K+1 (Eqs. 7, 10, 11).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void accept_kernel(const int32_t* __restrict__ draft, int draft_stride,
                                                    const int32_t* __restrict__ tgt,
                                                    const float* __restrict__ h_norm,
                                                    const int32_t* __restrict__ kv_len, int K,
                                                    float theta, int W,
                                                    int32_t* __restrict__ accept_len,
                                                    int32_t* __restrict__ next_token,
                                                    int32_t* __restrict__ n_loose,
                                                    int32_t* __restrict__ kv_len_out) {
  const int b = blockIdx.x, lane = threadIdx.x, j = lane + 1;
  const bool valid = j <= K;
  bool mism = false, strict = false;
  if (valid) {
    mism = draft[(int64_t)b * draft_stride + lane] != tgt[(int64_t)b * (K + 1) + lane];
    strict = h_norm[(int64_t)b * (K + 1) + lane] < theta;
  }
  const unsigned long long mm = __ballot(mism);  // bit l set: mismatch at position l+1
  bool rej = false;
  if (mism) {
    if (strict || W > K - j) {  // j + W > K, written so that no W overflows
      rej = true;
    } else if (W > 0) {
      // here j + W <= K <= 63, so both shifts are below 64
      unsigned long long win = ((1ull << W) - 1ull) << j;  // lanes j .. j+W-1 = positions j+1 .. j+W
      rej = (mm & win) != 0ull;
    }
  }
  const unsigned long long rb = __ballot(rej);
  if (lane == 0) {
    int s = rb ? __ffsll((long long)rb) : K + 1;
    accept_len[b] = s - 1;
    next_token[b] = tgt[(int64_t)b * (K + 1) + (s - 1)];
    if (n_loose != nullptr) n_loose[b] = __popcll(mm & ((1ull << (s - 1)) - 1ull));
    if (kv_len_out != nullptr && kv_len != nullptr) kv_len_out[b] = kv_len[b] + s;
  }
}

hipError_t launch_accept(const int32_t* draft, int draft_stride, const int32_t* tgt,
                         const float* h_norm, const int32_t* kv_len, int B, int K, float theta,
                         int W, int32_t* accept_len, int32_t* next_token, int32_t* n_loose,
                         int32_t* kv_len_out, hipStream_t st) {
  if (K < 1 || K > 63 || W < 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(64), 0, st, draft, draft_stride, tgt, h_norm, kv_len,
                     K, theta, W, accept_len, next_token, n_loose, kv_len_out);
  return hipGetLastError();
}
