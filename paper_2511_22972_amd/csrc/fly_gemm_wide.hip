// Weight-streaming bf16 GEMM for 129..256 activation rows (paper Sec. 2.1,
// Algorithm 1 step 2: the layer projections and the LM head of the
// verification forward when a batch of sequences is verified together, e.g.
// sixteen sequences with fifteen drafts each).
//
// In this range a GEMM of the forward is still bound by reading its weights
// once from HBM (256 flop per weight byte against ~310 at the ridge), but the
// accumulators of that many rows no longer fit the 16-row tiles of the kernel
// for small blocks, and staging the weights in LDS (the kernel for many rows)
// leaves too few weight bytes in flight per compute unit to keep HBM busy.
// Here every wave streams the packed weight tiles of its own 64 columns
// straight from global memory into matrix-core operand registers, through a
// ring of k-chunks that keeps 24-32 KiB per wave in flight, and only the small
// activation block is staged in LDS and shared by the four waves.  The product
// is out^T[n, m] = sum_k W[k, n] X[m, k] in 32 x 32 tiles of
// v_mfma_f32_32x32x16_bf16 (weights = A operand, activations = B operand); a
// wave holds 2 x MT of them (MT = 5, 6 or 8 tiles of 32 rows).
#include "fly_common.h"

typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr int WIDE_KC = 2;  // 32-wide k-tiles per chunk (pipeline step)

__device__ __forceinline__ float silu_w(float x) { return x / (1.f + __expf(-x)); }

// Softmax statistics of the 16 logits a lane holds of one 32 x 32 tile (columns
// n0 + 8 (r/4) + 4 hi + r%4 of one row), folded into the row's running statistics.
__device__ __forceinline__ void wide_row_stat(RowStat& run, const f32x16& v, float sc, int n0, int hi,
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

}  // namespace

// Grid: (column blocks of 256, split-K factor).
template <int MT, int EPI, int RING>
__global__ __launch_bounds__(256) void gemm_bf16_wide_kernel(
    const bf16_t* __restrict__ X, const u32x4* __restrict__ Wp, void* __restrict__ out,
    const float* __restrict__ row_scale, int M, int N, int Kd, int chunks_per_split, int nblocks) {
  constexpr int KC = WIDE_KC;
  // Workgroups are dealt to the eight XCDs round-robin by linear id; consecutive
  // column blocks go to different XCDs.
  const int nblock = blockIdx.x;
  if (nblock >= nblocks) return;

  // LDS: two stages of the activation block.  One k-tile (32 wide) of 16 rows is
  // 1 KiB: a row is four 16-byte pieces, piece c of row r at position
  // 4 r + (c ^ ((r >> 1) & 3)), so that the operand reads of eight consecutive
  // rows fall into distinct banks.
  __shared__ u32x4 xs[2][KC][2 * MT][64];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int ktiles = Kd / 32;
  const int nchunks_total = (ktiles + KC - 1) / KC;
  const int chunk_begin = blockIdx.y * chunks_per_split;
  const int chunk_end = min(chunk_begin + chunks_per_split, nchunks_total);
  const int kt_end = min(chunk_end * KC, ktiles);
  const int kt_last = max(kt_end - 1, 0);
  const int nstrips = N / 16;
  const int strip0 = nblock * 16 + wave * 4;  // this wave's four 16-column strips

  // Weight fragment (column group cg, k-tile kt, half kh) of the 32x32x16 A
  // operand: lane (l32, hi) holds W[32 kt + 16 kh + 8 hi + i][32 cg + l32],
  // i = 0..7, which in the packed layout is the 16-byte piece of lane
  // (l32 % 16) + 16 (hi + 2 kh) of the tile of strip 2 cg + l32 / 16.  Strips
  // past the last one (ragged last workgroup) are clamped: loaded and
  // multiplied like the others, never stored.  k-tiles at or past kt_end are
  // clamped to the last valid one; they meet zeroed activations.
  const u32x4* wbase[2];
#pragma unroll
  for (int cg = 0; cg < 2; ++cg) {
    const int strip = min(strip0 + 2 * cg + (l32 >> 4), nstrips - 1);
    wbase[cg] = Wp + (int64_t)strip * ktiles * 64 + (lane & 15) + 16 * hi;
  }
  auto load_w = [&](u32x4 (&a)[2][KC][2], int chunk) {
#pragma unroll
    for (int kt = 0; kt < KC; ++kt) {
      const int k = min(chunk * KC + kt, kt_last);
#pragma unroll
      for (int cg = 0; cg < 2; ++cg)
#pragma unroll
        for (int kh = 0; kh < 2; ++kh)
          a[cg][kt][kh] = __builtin_nontemporal_load(wbase[cg] + (int64_t)k * 64 + 32 * kh);
    }
  };

  // Activation pieces this wave stages per chunk: piece f = wave + 4 i is k-tile
  // f / (2 MT), row group f % (2 MT); lane 4 r + c' fetches row r of the group,
  // 16-byte piece c' ^ ((r >> 1) & 3), and writes it to position 4 r + c'.  Rows
  // past M are clamped to row M-1 (they feed output rows that are never
  // stored); k-tiles at or past kt_end read a clamped, valid address and are
  // replaced by zeros when written to LDS.
  constexpr int NXF = KC * 2 * MT / 4;
  static_assert(NXF * 4 == KC * 2 * MT, "activation pieces must divide evenly over the four waves");
  u32x4 xf[NXF];
  const bf16_t* xrow[NXF];
  int xkt[NXF], xgrp[NXF];
#pragma unroll
  for (int i = 0; i < NXF; ++i) {
    const int f = wave + 4 * i;
    xkt[i] = f / (2 * MT);
    xgrp[i] = f % (2 * MT);
    const int r = lane >> 2;
    const int piece = (lane & 3) ^ ((r >> 1) & 3);
    const int row = min(xgrp[i] * 16 + r, M - 1);
    xrow[i] = X + (int64_t)row * Kd + piece * 8;
  }
  auto load_x = [&](int chunk) {
#pragma unroll
    for (int i = 0; i < NXF; ++i) {
      const int k = min(chunk * KC + xkt[i], kt_last);
      xf[i] = *(const u32x4*)(xrow[i] + (int64_t)k * 32);
    }
  };
  auto store_x = [&](int stage, int chunk) {
#pragma unroll
    for (int i = 0; i < NXF; ++i) {
      u32x4 v = xf[i];
      if (chunk * KC + xkt[i] >= kt_end) v = u32x4{0u, 0u, 0u, 0u};
      xs[stage][xkt[i]][xgrp[i]][lane] = v;
    }
  };

  f32x16 acc[2][MT];
#pragma unroll
  for (int cg = 0; cg < 2; ++cg)
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[cg][t][r] = 0.f;

  // One chunk: for each 16-wide half of each k-tile, the MT activation
  // fragments (32 rows x 16 k each) come from LDS and meet the two weight
  // fragments of the wave.  The fragments of the next half are requested before
  // the multiplies of the current one.  The scheduling barriers pin that order:
  // left alone, the compiler moves each LDS read next to its first use (every
  // pair of multiplies then waits for a full LDS round trip) and sinks the
  // activation loads below the weight loads (writing them to LDS then waits for
  // the whole weight ring).
  auto read_b = [&](bf16x8 (&b)[MT], int stage, int kt, int kh) {
    const int r = l32 & 15;
    const int c = hi + 2 * kh;
#pragma unroll
    for (int t = 0; t < MT; ++t)
      b[t] = __builtin_bit_cast(bf16x8, xs[stage][kt][2 * t + (l32 >> 4)][4 * r + (c ^ ((r >> 1) & 3))]);
  };
  auto compute = [&](const u32x4 (&a)[2][KC][2], int stage) {
    bf16x8 b[2][MT];
    read_b(b[0], stage, 0, 0);
#pragma unroll
    for (int h = 0; h < 2 * KC; ++h) {
      const int kt = h >> 1, kh = h & 1;
      if (h + 1 < 2 * KC) read_b(b[(h + 1) & 1], stage, (h + 1) >> 1, (h + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int cg = 0; cg < 2; ++cg)
          acc[cg][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[cg][kt][kh]),
                                                               b[h & 1][t], acc[cg][t], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Software pipeline over k-chunks with a ring of RING weight buffers in
  // registers: while chunk c is multiplied, the weights of chunks c+1 ..
  // c+RING-1 are in flight.  The activation loads of chunk c+1 are issued before
  // the weight loads of chunk c+RING-1, so that writing them to LDS at the end
  // of the step waits only for them and the older weight loads (loads retire in
  // order).  Steps have no conditionals inside; the tail guards whole steps.
  u32x4 ring[RING][2][KC][2];
  int stage = 0;
  auto step = [&](const u32x4 (&cur)[2][KC][2], u32x4 (&refill)[2][KC][2], int chunk) {
    load_x(chunk + 1);
    __builtin_amdgcn_sched_barrier(0);
    load_w(refill, chunk + RING - 1);
    __builtin_amdgcn_sched_barrier(0);
    compute(cur, stage);
    store_x(stage ^ 1, chunk + 1);
    __syncthreads();
    stage ^= 1;
  };
  if (chunk_begin < chunk_end) {
    load_x(chunk_begin);
#pragma unroll
    for (int r = 0; r < RING - 1; ++r) load_w(ring[r], chunk_begin + r);
    store_x(0, chunk_begin);
    __syncthreads();
    int c = chunk_begin;
    while (c + RING <= chunk_end) {
#pragma unroll
      for (int r = 0; r < RING; ++r) step(ring[r], ring[(r + RING - 1) % RING], c + r);
      c += RING;
    }
#pragma unroll
    for (int r = 0; r < RING - 1; ++r)
      if (c + r < chunk_end) step(ring[r], ring[(r + RING - 1) % RING], c + r);
  }

  // ---- epilogues.  Accumulator register r of tile (cg, t) in lane l is
  // out^T[n = n0 + 32 cg + 8 (r/4) + 4 (l/32) + r%4][m = 32 t + l%32].
  const int n0 = strip0 * 16;
  if constexpr (EPI == EPI_PARTIAL) {
    float* o = (float*)out + (int64_t)blockIdx.y * M * N;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int m = t * 32 + l32;
      if (m >= M) continue;
#pragma unroll
      for (int cg = 0; cg < 2; ++cg) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + 32 * cg + 8 * q + 4 * hi;
          if (n < N) {
            f32x4 v = {acc[cg][t][4 * q], acc[cg][t][4 * q + 1], acc[cg][t][4 * q + 2], acc[cg][t][4 * q + 3]};
            *(f32x4*)(o + (int64_t)m * N + n) = v;
          }
        }
      }
    }
  } else if constexpr (EPI == EPI_SWIGLU) {
    // strips alternate gate / up: rows 0..15 of a 32-row tile are gate columns,
    // rows 16..31 the matching up columns (registers r and r + 8).
    bf16_t* o = (bf16_t*)out;
    const int Nh = N / 2;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int m = t * 32 + l32;
      if (m >= M) continue;
#pragma unroll
      for (int cg = 0; cg < 2; ++cg) {
        if (n0 + 32 * cg + 31 >= N) continue;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          float a0 = silu_w(acc[cg][t][4 * q + 0]) * acc[cg][t][4 * q + 8];
          float a1 = silu_w(acc[cg][t][4 * q + 1]) * acc[cg][t][4 * q + 9];
          float a2 = silu_w(acc[cg][t][4 * q + 2]) * acc[cg][t][4 * q + 10];
          float a3 = silu_w(acc[cg][t][4 * q + 3]) * acc[cg][t][4 * q + 11];
          u32x2 pk;
          pk.x = pack_bf2(a0, a1);
          pk.y = pack_bf2(a2, a3);
          *(u32x2*)(o + (int64_t)m * Nh + (n0 + 32 * cg) / 2 + 8 * q + 4 * hi) = pk;
        }
      }
    }
  } else {  // EPI_LMHEAD: softmax statistics of this wave's 64 columns per row
    f32x4* o = (f32x4*)out;
    const int nparts = nblocks * 4;
    const int part = nblock * 4 + wave;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int m = t * 32 + l32;
      const float sc = (row_scale != nullptr && m < M) ? row_scale[m] : 1.f;
      RowStat st = stat_empty();
#pragma unroll
      for (int cg = 0; cg < 2; ++cg) wide_row_stat(st, acc[cg][t], sc, n0 + 32 * cg, hi, N);
      st = stat_merge(st, stat_shfl_xor(st, 32));
      if (hi == 0 && m < M) {
        f32x4 w;
        w.x = st.m;
        w.y = st.s;
        w.z = st.t;
        w.w = __int_as_float(st.idx);
        o[(int64_t)m * nparts + part] = w;
      }
    }
  }
}

template <int MT, int RING>
static hipError_t launch_wide_mt(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale, int M,
                                 int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st) {
  const int nblocks = (N / 16 + 15) / 16;
  const int nchunks = (Kd / 32 + WIDE_KC - 1) / WIDE_KC;
  const int cps = (nchunks + plan.splits - 1) / plan.splits;
  dim3 grid(nblocks, plan.splits, 1), block(256);
  const u32x4* W4 = (const u32x4*)Wp;
  if (epi == EPI_PARTIAL)
    hipLaunchKernelGGL((gemm_bf16_wide_kernel<MT, EPI_PARTIAL, RING>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks);
  else if (epi == EPI_SWIGLU)
    hipLaunchKernelGGL((gemm_bf16_wide_kernel<MT, EPI_SWIGLU, RING>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks);
  else
    hipLaunchKernelGGL((gemm_bf16_wide_kernel<MT, EPI_LMHEAD, RING>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks);
  return hipGetLastError();
}

// plan.wide = number of 32-row tiles (5, 6 or 8).
hipError_t launch_gemm_bf16_wide(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale, int M,
                                 int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st) {
  // Host-side shape checks: whole 16-column tiles and 32-row k-tiles, all rows
  // inside the one row block, every split owning at least one chunk.
  if (N % 16 != 0 || Kd % 32 != 0 || M < 1 || M > plan.wide * 32) return hipErrorInvalidValue;
  if (epi != EPI_PARTIAL && epi != EPI_SWIGLU && epi != EPI_LMHEAD) return hipErrorInvalidValue;
  if (plan.splits < 1 || (epi != EPI_PARTIAL && plan.splits != 1)) return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU && N % 32 != 0) return hipErrorInvalidValue;
  const int nchunks = (Kd / 32 + WIDE_KC - 1) / WIDE_KC;
  const int cps = (nchunks + plan.splits - 1) / plan.splits;
  if ((plan.splits - 1) * cps >= nchunks) return hipErrorInvalidValue;
  switch (plan.wide) {
    case 5: return launch_wide_mt<5, 5>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st);
    case 6: return launch_wide_mt<6, 5>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st);
    case 8: return launch_wide_mt<8, 4>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st);
  }
  return hipErrorInvalidValue;
}

int gemm_bf16_wide_lmhead_parts(int N) { return (N / 16 + 15) / 16 * 4; }
