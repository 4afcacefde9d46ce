// Weight packing and the weight-streaming GEMMs of the verification forward
// (layer projections and the LM head; paper Sec. 2.1, Algorithm 1 step 2).
//
// The block of K+1 draft positions gives M = B*(K+1) activation rows, a few
// dozen, against weight matrices of 10^8..10^9 entries, so every GEMM here is
// bound by reading the weights once from HBM.  The bf16 kernel therefore
// streams packed weight tiles straight from global memory into matrix-core
// operand registers (each wave-level load is one contiguous KiB), keeps the
// small activation block in LDS in operand order, and computes
// out^T[n, m] = sum_k W[k, n] X[m, k] with v_mfma_f32_16x16x32_bf16 so that the
// weight tile is the A operand and the activations are the B operand.
#include "fly_common.h"

// ---------------------------------------------------------------------------
// Packing
// ---------------------------------------------------------------------------
// bf16 packed layout: tile (tn, tk) covers columns 16tn..16tn+15 and rows
// 32tk..32tk+31 of W[k_in, n]; it occupies 64 lanes x 8 values, lane l holding
// W[32tk + 8(l/16) + i][16tn + l%16], i = 0..7.  Tiles of one column strip are
// contiguous along tk.
__global__ void pack_bf16_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst,
                                 int64_t k_in, int64_t n_src, int64_t tile_offset,
                                 int64_t tile_stride) {
  int64_t ktiles = k_in / 32;
  int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one (tile, lane) each
  int64_t total = (n_src / 16) * ktiles * 64;
  if (gid >= total) return;
  int lane = (int)(gid % 64);
  int64_t tile = gid / 64;
  int64_t tk = tile % ktiles;
  int64_t tj = tile / ktiles;  // source column tile
  int64_t tn = tile_offset + tj * tile_stride;
  int64_t col = tj * 16 + (lane & 15);
  int64_t row0 = tk * 32 + 8 * (lane >> 4);
  bf16_t v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = src[(row0 + i) * n_src + col];
  bf16_t* d = dst + ((tn * ktiles + tk) * 64 + lane) * 8;
#pragma unroll
  for (int i = 0; i < 8; ++i) d[i] = v[i];
}

__global__ void pack_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t k_in,
                                int64_t n_src, int64_t n_dst, int64_t tile_offset,
                                int64_t tile_stride) {
  int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= k_in * n_src) return;
  int64_t k = gid / n_src, c = gid % n_src;
  int64_t tn = tile_offset + (c / 16) * tile_stride;
  dst[k * n_dst + tn * 16 + (c & 15)] = src[gid];
}

hipError_t launch_pack_weight(const void* src, int64_t k_in, int64_t n_src, int dtype, void* dst,
                              int64_t n_dst, int64_t tile_offset, int64_t tile_stride,
                              hipStream_t st) {
  if (dtype == FLY_BF16) {
    int64_t total = (n_src / 16) * (k_in / 32) * 64;
    int64_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(pack_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                       (const bf16_t*)src, (bf16_t*)dst, k_in, n_src, tile_offset, tile_stride);
  } else {
    int64_t total = k_in * n_src;
    int64_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(pack_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const float*)src,
                       (float*)dst, k_in, n_src, n_dst, tile_offset, tile_stride);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// bf16 weight-streaming GEMM
// ---------------------------------------------------------------------------
// KS = 32-wide k-steps per pipeline stage: 4 (128 k) normally, 2 for the nine-row-tile variant,
// whose accumulators leave less room for the prefetch ring.

__device__ __forceinline__ float silu_f(float x) { return x / (1.f + __expf(-x)); }

template <int MT, int NT>
struct GemmRegs {
  f32x4 acc[NT][MT];
};

// Issue the global loads of one k-chunk: NT x KS weight tiles for this wave.
// Always unconditional (so that all loads of a chunk are in flight together and
// the loop around it has no branches): k-steps past the end of this workgroup's
// range are clamped to its last k-step.  They load valid weights that are then
// multiplied by zero activations.
template <int NT, int KS, bool CLAMP>
__device__ __forceinline__ void load_weight_chunk(u32x4 (&a)[NT][KS], const u32x4* const (&wstrip)[NT],
                                                  int ks0, int ks_last, int lane) {
#pragma unroll
  for (int j = 0; j < NT; ++j) {
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int ks = CLAMP ? min(ks0 + s, ks_last) : ks0 + s;
      a[j][s] = __builtin_nontemporal_load(wstrip[j] + (int64_t)ks * 64 + lane);
    }
  }
}

template <int MT, int NT, int EPI, int KS, int RING>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(
    const bf16_t* __restrict__ X, const u32x4* __restrict__ Wp, void* __restrict__ out,
    const float* __restrict__ row_scale, int M, int N, int Kd, int chunks_per_split, int nblocks,
    int mblocks, LmSample smp) {
  // Workgroup -> (column block, row block).  Workgroups are dealt to the eight
  // XCDs (each with its own L2) round-robin by linear id.  When the activations
  // need several row blocks, the row blocks of one column block re-read the same
  // weight strips: they are given consecutive slots of ONE XCD so that they run
  // together and all but the first find the strips in that XCD's L2.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int mblock = slot % mblocks;
  const int nblock = (slot / mblocks) * 8 + xcd;
  if (nblock >= nblocks) return;  // padding of the last group of eight (uniform per workgroup)
  // LDS: two stages of the activation block in operand order
  // [stage][kstep][mtile][lane] x 16 bytes.
  constexpr int NFRAG_W = (KS * MT + 3) / 4;  // fragments each wave stages per chunk
  __shared__ u32x4 xs[2][NFRAG_W * 4][64];   // fragment f = kstep * MT + row tile (padded to 4 per wave)

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: uniform branches
  const int g = lane >> 4, c16 = lane & 15;
  const int ksteps_total = Kd / 32;
  const int nchunks_total = (ksteps_total + KS - 1) / KS;
  const int chunk_begin = blockIdx.y * chunks_per_split;
  int chunk_end = chunk_begin + chunks_per_split;
  if (chunk_end > nchunks_total) chunk_end = nchunks_total;
  const int ks_end = min(chunk_end * KS, ksteps_total);
  const int ks_last = max(ks_end - 1, 0);
  const int mrow0 = mblock * (MT * 16);
  const int ntiles = N / 16;
  const int tn0 = (nblock * 4 + wave) * NT;

  // Column strips of this wave.  A strip past the last tile (ragged last
  // workgroup) is clamped to the last tile: it is loaded and multiplied like the
  // others, and simply not stored.
  bool tile_ok[NT];
  const u32x4* wstrip[NT];
  const int64_t strip_stride = (int64_t)ksteps_total * 64;  // u32x4 units per column strip
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    tile_ok[j] = (tn0 + j) < ntiles;
    wstrip[j] = Wp + (int64_t)min(tn0 + j, ntiles - 1) * strip_stride;
  }

  f32x4 acc[NT][MT];
#pragma unroll
  for (int j = 0; j < NT; ++j)
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[j][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Activation fragments this wave stages per chunk: f = wave + 4i (k-step f / MT,
  // row tile f % MT).  Fragment indices past KS*MT (padding, when KS*MT is not a
  // multiple of 4) reload the last fragment into a padding slot nobody reads, which
  // keeps the loop branch-free.  Rows past M are clamped to row M-1: they only
  // feed output rows that are never stored.
  u32x4 xf[NFRAG_W];
  const bf16_t* xrow[NFRAG_W];
  int xks[NFRAG_W];
#pragma unroll
  for (int i = 0; i < NFRAG_W; ++i) {
    int f = min(wave + 4 * i, KS * MT - 1);
    int row = min(mrow0 + (f % MT) * 16 + c16, M - 1);
    xks[i] = f / MT;
    xrow[i] = X + (int64_t)row * Kd + xks[i] * 32 + 8 * g;
  }
  // k-steps at or past ks_end (ragged last chunk, or the up to two surplus
  // pipeline steps) read a clamped, valid address; they are replaced by zeros
  // when written to LDS (not at load time, which would wait for the load).
  auto load_x = [&](int chunk) {
#pragma unroll
    for (int i = 0; i < NFRAG_W; ++i) {
      const int kc = min(chunk * KS + xks[i], ks_last) - xks[i];  // xrow already points at k-step xks[i]
      xf[i] = *(const u32x4*)(xrow[i] + (int64_t)kc * 32);
    }
  };
  // the same for a chunk known to lie wholly inside the range
  auto load_x_inner = [&](int chunk) {
#pragma unroll
    for (int i = 0; i < NFRAG_W; ++i) xf[i] = *(const u32x4*)(xrow[i] + (int64_t)chunk * (KS * 32));
  };
  auto store_x = [&](int stage, int chunk) {  // chunk < 0: no masking needed
#pragma unroll
    for (int i = 0; i < NFRAG_W; ++i) {
      u32x4 v = xf[i];
      if (chunk >= 0 && chunk * KS + xks[i] >= ks_end) v = u32x4{0u, 0u, 0u, 0u};
      xs[stage][wave + 4 * i][lane] = v;
    }
  };

  // All activation fragments of the chunk are requested from LDS up front, so
  // that the reads are in flight together and only the first multiply waits
  // for LDS latency (issued pairwise just before use, each pair stalls the
  // matrix pipe for a full LDS round trip).
  auto compute = [&](const u32x4 (&a)[NT][KS], int stage) {
    u32x4 bfrag[KS][MT];
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int t = 0; t < MT; ++t) bfrag[s][t] = xs[stage][s * MT + t][lane];
    __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the multiplies
#pragma unroll
    for (int s = 0; s < KS; ++s) {
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        bf16x8 b = __builtin_bit_cast(bf16x8, bfrag[s][t]);
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          bf16x8 av = __builtin_bit_cast(bf16x8, a[j][s]);
          acc[j][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, b, acc[j][t], 0, 0, 0);
        }
      }
    }
    // ... and the LDS write of the next chunk's activations (which waits for their
    // global loads) behind the multiplies
    __builtin_amdgcn_sched_barrier(0);
  };

  // Software pipeline over k-chunks with a ring of RING weight buffers in
  // registers: while chunk c is multiplied, the weights of chunks c+1 ..
  // c+RING-1 are in flight (the bytes in flight per compute unit are what
  // decides the achieved HBM bandwidth).  The activation loads of chunk c+1 are
  // issued BEFORE the weight loads of chunk c+RING-1, so that writing them to
  // LDS at the end of the step waits only for them (loads retire in order) and
  // leaves the weight loads in flight.  Step bodies have no conditionals -- with
  // branches in them the compiler waits for every outstanding load before each
  // multiply and keeps a second copy of the accumulators; the tail guards whole
  // steps instead.
  u32x4 ring[RING][NT][KS];
  int stage = 0;

  if (chunk_begin < chunk_end) {
    load_x(chunk_begin);
#pragma unroll
    for (int r = 0; r < RING - 1; ++r)
      load_weight_chunk<NT, KS, true>(ring[r], wstrip, (chunk_begin + r) * KS, ks_last, lane);
    store_x(0, chunk_begin);
    __syncthreads();
    int c = chunk_begin;
    // steady state: every chunk touched (up to c + 2 RING - 2) lies wholly inside
    // the range, so addresses are plain base + offset
    const int inner_end = ks_end / KS;  // chunks below this index are complete
    while (c + 2 * RING - 2 < inner_end) {
#pragma unroll
      for (int r = 0; r < RING; ++r) {
        load_x_inner(c + r + 1);
        load_weight_chunk<NT, KS, false>(ring[(r + RING - 1) % RING], wstrip, (c + r + RING - 1) * KS, ks_last, lane);
        compute(ring[r], stage);
        store_x(stage ^ 1, -1);
        __syncthreads();
        stage ^= 1;
      }
      c += RING;
    }
    // last few chunks: clamped addresses, zero activations past the end
    for (; c < chunk_end; c += RING) {
#pragma unroll
      for (int r = 0; r < RING; ++r) {
        if (r == 0 || c + r < chunk_end) {
          load_x(c + r + 1);
          load_weight_chunk<NT, KS, true>(ring[(r + RING - 1) % RING], wstrip, (c + r + RING - 1) * KS, ks_last, lane);
          compute(ring[r], stage);
          store_x(stage ^ 1, c + r + 1);
          __syncthreads();
          stage ^= 1;
        }
      }
    }
  }

  // ---- epilogues.  Lane holds out^T[n = 16*tile + 4g + r][m = 16t + c16], r = 0..3.
  if constexpr (EPI == EPI_PARTIAL) {
    float* o = (float*)out + (int64_t)blockIdx.y * M * N;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      if (!tile_ok[j]) continue;
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        int m = mrow0 + t * 16 + c16;
        if (m < M) *(f32x4*)(o + (int64_t)m * N + (tn0 + j) * 16 + 4 * g) = acc[j][t];
      }
    }
  } else if constexpr (EPI == EPI_SWIGLU) {
    // column tiles alternate gate / up; output column = 16*(tile/2) + 4g + r
    bf16_t* o = (bf16_t*)out;
    const int Nh = N / 2;
#pragma unroll
    for (int j = 0; j + 1 < NT; j += 2) {
      if (!tile_ok[j + 1]) continue;
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        int m = mrow0 + t * 16 + c16;
        if (m < M) {
          f32x4 gt = acc[j][t], up = acc[j + 1][t];
          u32x2 pk;
          pk.x = pack_bf2(silu_f(gt.x) * up.x, silu_f(gt.y) * up.y);
          pk.y = pack_bf2(silu_f(gt.z) * up.z, silu_f(gt.w) * up.w);
          *(u32x2*)(o + (int64_t)m * Nh + ((tn0 + j) / 2) * 16 + 4 * g) = pk;
        }
      }
    }
  } else {  // EPI_LMHEAD / EPI_LMSAMPLE: per-wave softmax statistics of this wave's columns
    f32x4* o = (f32x4*)out;
    const int nparts = nblocks * 4;
    const int part = nblock * 4 + wave;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      int m = mrow0 + t * 16 + c16;
      float sc = (row_scale != nullptr && m < M) ? row_scale[m] : 1.f;
      float v[NT][4];
      float mx = -INFINITY;
      int idx = 0x7fffffff;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          v[j][r] = acc[j][t][r] * sc;
          if (tile_ok[j] && v[j][r] > mx) {
            mx = v[j][r];
            idx = (tn0 + j) * 16 + 4 * g + r;
          }
        }
      }
      RowStat st = stat_empty();
      if (idx != 0x7fffffff) {
        st.m = mx;
        st.idx = idx;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          if (!tile_ok[j]) continue;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float dlt = v[j][r] - mx;
            float e = __expf(dlt);
            st.s += e;
            st.t += dlt * e;
          }
        }
      }
      st = stat_merge(st, stat_shfl_xor(st, 16));
      st = stat_merge(st, stat_shfl_xor(st, 32));
      if (g == 0 && m < M) {
        f32x4 w;
        w.x = st.m;
        w.y = st.s;
        w.z = st.t;
        w.w = __int_as_float(st.idx);
        o[(int64_t)m * nparts + part] = w;
      }
      if constexpr (EPI == EPI_LMSAMPLE) {
        // the drawn token: largest Gumbel-perturbed logit of this wave's columns
        RowPick pk = pick_empty();
#pragma unroll
        for (int j = 0; j < NT; ++j)
          if (tile_ok[j])
            pick_update4(pk, v[j][0], v[j][1], v[j][2], v[j][3], (tn0 + j) * 16 + 4 * g, m, smp);
        pk = pick_merge(pk, pick_shfl_xor(pk, 16));
        pk = pick_merge(pk, pick_shfl_xor(pk, 32));
        if (g == 0 && m < M) pick_store(smp, (int64_t)m * nparts + part, pk);
      }
    }
  }
}

template <int MT, int NT>
static hipError_t launch_gemm_mt_nt(const bf16_t* X, const bf16_t* Wp, void* out,
                                    const float* row_scale, int M, int N, int Kd,
                                    const GemmPlan& plan, int epi, hipStream_t st, const LmSample& smp) {
  constexpr int KS = MT >= 9 ? 2 : 4;
  constexpr int RING = MT >= 9 ? 4 : 3;  // the same bytes in flight with half-size chunks
  int ntiles = N / 16;
  int nblocks = (ntiles + 4 * NT - 1) / (4 * NT);
  int nchunks = (Kd / 32 + KS - 1) / KS;
  int cps = (nchunks + plan.splits - 1) / plan.splits;
  dim3 grid((nblocks + 7) / 8 * 8 * plan.mblocks, plan.splits, 1), block(256);
  const u32x4* W4 = (const u32x4*)Wp;
  if (epi == EPI_PARTIAL) {
    hipLaunchKernelGGL((gemm_bf16_kernel<MT, NT, EPI_PARTIAL, KS, RING>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks, plan.mblocks, smp);
  } else if (epi == EPI_SWIGLU) {
    if constexpr (NT >= 2) {
      hipLaunchKernelGGL((gemm_bf16_kernel<MT, NT, EPI_SWIGLU, KS, RING>), grid, block, 0, st, X, W4, out,
                         row_scale, M, N, Kd, cps, nblocks, plan.mblocks, smp);
    } else {
      return hipErrorInvalidValue;
    }
  } else if (epi == EPI_LMHEAD) {
    hipLaunchKernelGGL((gemm_bf16_kernel<MT, NT, EPI_LMHEAD, KS, RING>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks, plan.mblocks, smp);
  } else {
    hipLaunchKernelGGL((gemm_bf16_kernel<MT, NT, EPI_LMSAMPLE, KS, RING>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks, plan.mblocks, smp);
  }
  return hipGetLastError();
}

template <int MT>
static hipError_t launch_gemm_mt(const bf16_t* X, const bf16_t* Wp, void* out,
                                 const float* row_scale, int M, int N, int Kd, const GemmPlan& plan,
                                 int epi, hipStream_t st, const LmSample& smp) {
  switch (plan.nt) {
    case 1: return launch_gemm_mt_nt<MT, 1>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 2: return launch_gemm_mt_nt<MT, 2>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 4: return launch_gemm_mt_nt<MT, 4>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_gemm_bf16(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale,
                            int M, int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st,
                            const LmSample& smp) {
  if (epi < EPI_PARTIAL || epi > EPI_LMSAMPLE) return hipErrorInvalidValue;
  if (epi == EPI_LMSAMPLE && smp.pick == nullptr) return hipErrorInvalidValue;
  if (plan.wide) return launch_gemm_bf16_wide(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
  if (plan.tiled) return launch_gemm_bf16_tiled(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
  // Host-side shape checks: the kernel assumes whole 16-column tiles and whole
  // 32-row k-steps, and that the row blocks cover M.
  if (N % 16 != 0 || Kd % 32 != 0 || M < 1) return hipErrorInvalidValue;
  if (plan.mblocks * plan.mt * 16 < M) return hipErrorInvalidValue;
  if (epi != EPI_PARTIAL && plan.splits != 1) return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU && (N % 32 != 0)) return hipErrorInvalidValue;
  switch (plan.mt) {
    case 1: return launch_gemm_mt<1>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 2: return launch_gemm_mt<2>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 3: return launch_gemm_mt<3>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 5: return launch_gemm_mt<5>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 9: return launch_gemm_mt<9>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
  }
  return hipErrorInvalidValue;
}

int gemm_bf16_lmhead_parts(int N, const GemmPlan& plan) {
  if (plan.wide) return gemm_bf16_wide_lmhead_parts(N);
  if (plan.tiled) return gemm_bf16_tiled_lmhead_parts(N, plan.tiled);
  int ntiles = N / 16;
  int nblocks = (ntiles + 4 * plan.nt - 1) / (4 * plan.nt);
  return nblocks * 4;
}

// ---------------------------------------------------------------------------
// fp32 GEMM (tiny configuration): block = 64 columns x 16 k-slices, up to 8 rows.
// The shapes are a few hundred wide, so the kernel is bound by the latency of
// its k loop: sixteen slices keep the loop short, the slices are added in
// slice order (the result does not depend on scheduling).
// ---------------------------------------------------------------------------
#define F32_MB 8
#define F32_KSL 16

template <int EPI>
__global__ __launch_bounds__(64 * F32_KSL) void gemm_f32_kernel(const float* __restrict__ X,
                                                                const float* __restrict__ W,
                                                                void* __restrict__ out,
                                                                const float* __restrict__ row_scale,
                                                                int M, int N, int Kd, LmSample smp) {
  __shared__ float red[F32_KSL][F32_MB][64];
  const int c = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + c;
  const int m0 = blockIdx.y * F32_MB;
  float acc[F32_MB];
#pragma unroll
  for (int r = 0; r < F32_MB; ++r) acc[r] = 0.f;
  if (n < N) {
    // unrolled so that several weight loads are in flight; the additions stay in k order
#pragma unroll 4
    for (int k = slice; k < Kd; k += F32_KSL) {
      float w = W[(int64_t)k * N + n];
#pragma unroll
      for (int r = 0; r < F32_MB; ++r) {
        int m = m0 + r;
        float x = (m < M) ? X[(int64_t)m * Kd + k] : 0.f;
        acc[r] = fmaf(x, w, acc[r]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < F32_MB; ++r) red[slice][r][c] = acc[r];
  __syncthreads();
  // thread (slice, c) with slice < 8 finishes row `slice` of column c: it alone
  // reads and rewrites that row's entries
  const int r = slice, m = m0 + r;
  if (slice < F32_MB) {
    float t = red[0][r][c];
#pragma unroll
    for (int s = 1; s < F32_KSL; ++s) t += red[s][r][c];
    red[0][r][c] = t;
  }
  __syncthreads();
  if (slice >= F32_MB) return;
  if constexpr (EPI == EPI_PARTIAL) {
    float* o = (float*)out;
    if (m < M && n < N) o[(int64_t)m * N + n] = red[0][r][c];
  } else if constexpr (EPI == EPI_SWIGLU) {
    // 16-column tiles alternate gate / up inside the 64-column block
    float* o = (float*)out;
    const int Nh = N / 2;
    if (c < 32) {  // pair 0 uses tiles (0,1), pair 1 tiles (2,3) of this block
      const int pair = c >> 4, e = c & 15;
      int ncol = blockIdx.x * 64 + pair * 32 + e;  // gate column in the packed matrix
      if (m < M && ncol + 16 < N) {
        float gt = red[0][r][pair * 32 + e], up = red[0][r][pair * 32 + 16 + e];
        o[(int64_t)m * Nh + blockIdx.x * 32 + pair * 16 + e] = silu_f(gt) * up;
      }
    }
  } else {
    f32x4* o = (f32x4*)out;
    const int nparts = gridDim.x;
    float sc = (row_scale != nullptr && m < M) ? row_scale[m] : 1.f;
    RowStat st = stat_empty();
    if (n < N) {
      st.m = red[0][r][c] * sc;
      st.s = 1.f;
      st.t = 0.f;
      st.idx = n;
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) st = stat_merge(st, stat_shfl_xor(st, off));
    if (c == 0 && m < M) {
      f32x4 w;
      w.x = st.m;
      w.y = st.s;
      w.z = st.t;
      w.w = __int_as_float(st.idx);
      o[(int64_t)m * nparts + blockIdx.x] = w;
    }
    if constexpr (EPI == EPI_LMSAMPLE) {
      RowPick pk = n < N ? pick_one(red[0][r][c] * sc, n, m, smp) : pick_empty();
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) pk = pick_merge(pk, pick_shfl_xor(pk, off));
      if (c == 0 && m < M) pick_store(smp, (int64_t)m * nparts + blockIdx.x, pk);
    }
  }
}

hipError_t launch_gemm_f32(const float* X, const float* W, void* out, const float* row_scale, int M,
                           int N, int Kd, int epi, hipStream_t st, const LmSample& smp) {
  if (N % 16 != 0 || M < 1 || Kd < 1) return hipErrorInvalidValue;
  if (epi < EPI_PARTIAL || epi > EPI_LMSAMPLE) return hipErrorInvalidValue;
  if (epi == EPI_LMSAMPLE && smp.pick == nullptr) return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU && N % 32 != 0) return hipErrorInvalidValue;
  dim3 grid((N + 63) / 64, (M + F32_MB - 1) / F32_MB), block(64 * F32_KSL);
  if (epi == EPI_PARTIAL)
    hipLaunchKernelGGL((gemm_f32_kernel<EPI_PARTIAL>), grid, block, 0, st, X, W, out, row_scale, M, N, Kd, smp);
  else if (epi == EPI_SWIGLU)
    hipLaunchKernelGGL((gemm_f32_kernel<EPI_SWIGLU>), grid, block, 0, st, X, W, out, row_scale, M, N, Kd, smp);
  else if (epi == EPI_LMHEAD)
    hipLaunchKernelGGL((gemm_f32_kernel<EPI_LMHEAD>), grid, block, 0, st, X, W, out, row_scale, M, N, Kd, smp);
  else
    hipLaunchKernelGGL((gemm_f32_kernel<EPI_LMSAMPLE>), grid, block, 0, st, X, W, out, row_scale, M, N, Kd, smp);
  return hipGetLastError();
}

int gemm_f32_lmhead_parts(int N) { return (N + 63) / 64; }
