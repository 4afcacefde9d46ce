// Weight-streaming bf16 GEMM for 81..256 activation rows (paper Sec. 2.1,
// Algorithm 1 step 2: the layer projections and the LM head of the
// verification forward when a batch of sequences is verified together, e.g.
// sixteen sequences with fifteen drafts each).
//
// In this range a GEMM of the forward is still bound by reading its weights
// once from HBM (256 flop per weight byte against ~310 at the ridge), but the
// matrix work is no longer small beside it, the accumulators of that many rows
// do not fit the 16-row tiles of the kernel for small blocks, and staging the
// weights in LDS (the kernel for many rows) leaves too few weight bytes in
// flight per compute unit to keep HBM busy.  Here a workgroup of eight waves
// covers 256 columns: every wave streams the packed weight tiles of its own 32
// columns straight from global memory into matrix-core operand registers,
// through a ring of k-chunks, and holds MT accumulator tiles of
// v_mfma_f32_32x32x16_bf16 (MT = 3, 4, 5, 6 or 8 tiles of 32 rows; weights = A
// operand, activations = B operand, out^T[n, m] = sum_k W[k, n] X[m, k]).  Two
// waves share a SIMD, so one multiplies while the other waits for its weights.
// Only the small activation block goes through LDS: every wave fetches its
// share of it into registers two chunks ahead and writes it to LDS one chunk
// ahead.  All loads of the kernel are ordinary register loads, so the compiler
// places every wait.  (An earlier form copied the activations with LDS-direct
// loads and counted the waits by hand, assuming that a wave's LDS-direct loads
// and its register loads complete in issue order relative to each other.  They do
// not on this chip: with activations that miss the L2 -- the down projection at the
// 405B width -- about one launch in twelve read an activation stage that had not
// landed yet.)
#include "fly_common.h"

std::atomic<int> g_wide_phase{0};  // tuning knob: 0 automatic, 1 half of the waves late, 2 every wave early

namespace {

constexpr int WIDE_KC = 2;  // 32-wide k-tiles per chunk (pipeline step)
constexpr int WIDE_NWV = 8;  // waves per workgroup
constexpr int WIDE_CG = 1;   // 32-column groups per wave
constexpr int WIDE_COLS = 32 * WIDE_CG * WIDE_NWV;

__device__ __forceinline__ float silu_w(float x) { return x / (1.f + __expf(-x)); }

}  // namespace

// Grid: (column blocks of 256, split-K factor).
// NWV waves per workgroup, each owning CG groups of 32 columns: a workgroup covers
// 32 CG NWV columns.
template <int MT, int EPI, int RING, int NWV, int CG>
__global__ __launch_bounds__(64 * NWV) void gemm_bf16_wide_kernel(
    const bf16_t* __restrict__ X, const u32x4* __restrict__ Wp, void* __restrict__ out,
    const float* __restrict__ row_scale, int M, int N, int Kd, int chunks_per_split, int nblocks,
    int phase, LmSample smp) {
  constexpr int KC = WIDE_KC;
  constexpr int WGS = 2 * CG * NWV;  // 16-column strips per workgroup
  // Workgroups are dealt to the eight XCDs round-robin by linear id; consecutive
  // column blocks go to different XCDs.
  const int nblock = blockIdx.x;
  if (nblock >= nblocks) return;

  // LDS: two activation blocks (the one being multiplied, the one being written).
  // One k-tile (32 wide) of 16 rows is 1 KiB: a row is four 16-byte pieces, piece c
  // of row r at position 4 r + (c ^ ((r >> 2) & 3)): a 128-bit LDS read serves
  // sixteen lanes per cycle -- lanes 0-7 together with 24-31, 8-15 with 16-23, the same
  // in the upper half-wave (measured) --, and the sixteen rows such a set reads (rows
  // 0-7 of one 16-row group, 8-15 of the next) then fall into sixteen distinct phases.
  static_assert(RING % 2 == 0, "the register buffers of the activations alternate with the ring");
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
  const int strip0 = nblock * WGS + wave * (2 * CG);  // this wave's 16-column strips (two per column group)

  // Weight fragment (column group cg, k-tile kt, half kh) of the 32x32x16 A
  // operand: lane (l32, hi) holds W[32 kt + 16 kh + 8 hi + i][32 cg + l32],
  // i = 0..7, which in the packed layout is the 16-byte piece of lane
  // (l32 % 16) + 16 (hi + 2 kh) of the tile of strip 2 cg + l32 / 16.  Strips
  // past the last one (ragged last workgroup) are clamped: loaded and
  // multiplied like the others, never stored.  k-tiles at or past kt_end (ragged
  // last chunk, surplus pipeline steps) are clamped to the last valid one and
  // the fragment is replaced by zeros once loaded.
  const u32x4* wbase[CG];
#pragma unroll
  for (int cg = 0; cg < CG; ++cg) {
    const int strip = min(strip0 + 2 * cg + (l32 >> 4), nstrips - 1);
    wbase[cg] = Wp + (int64_t)strip * ktiles * 64 + (lane & 15) + 16 * hi;
  }
  auto load_w_kt = [&](u32x4 (&a)[CG][KC][2], int chunk, int kt) {
    const int k = min(chunk * KC + kt, kt_last);
#pragma unroll
    for (int cg = 0; cg < CG; ++cg)
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
        a[cg][kt][kh] = __builtin_nontemporal_load(wbase[cg] + (int64_t)k * 64 + 32 * kh);
  };
  auto load_w = [&](u32x4 (&a)[CG][KC][2], int chunk) {
#pragma unroll
    for (int kt = 0; kt < KC; ++kt) load_w_kt(a, chunk, kt);
  };

  // Activation pieces this wave copies per chunk: piece f = wave + NWV i is k-tile
  // f / (2 MT), row group f % (2 MT); lane 4 r + c' fetches row r of the group,
  // 16-byte piece c' ^ ((r >> 2) & 3), and the wave's 1 KiB is stored in lane
  // order.  Rows past M are clamped to row M-1 (they feed output rows that are
  // never stored), k-tiles past the end to the last valid one (they meet zeroed
  // weight fragments).  A wave whose last piece index falls past the block loads
  // the last piece again and does not store it (the loads stay unconditional so that
  // the compiler can count exactly how many were issued after the one it waits for).
  constexpr int NPIECE = KC * 2 * MT;
  constexpr int NXL = (NPIECE + NWV - 1) / NWV;
  const u32x4* xrow[NXL];
  int xkt[NXL], xgrp[NXL];
#pragma unroll
  for (int i = 0; i < NXL; ++i) {
    const int fc = min(wave + NWV * i, NPIECE - 1);
    xkt[i] = fc / (2 * MT);
    xgrp[i] = fc % (2 * MT);
    const int r = lane >> 2;
    const int piece = (lane & 3) ^ ((r >> 2) & 3);
    const int row = min(xgrp[i] * 16 + r, M - 1);
    xrow[i] = (const u32x4*)(X + (int64_t)row * Kd + piece * 8);
  }
  auto load_x = [&](u32x4 (&xb)[NXL], int chunk) {
#pragma unroll
    for (int i = 0; i < NXL; ++i) {
      const int k = min(chunk * KC + xkt[i], kt_last);
      xb[i] = xrow[i][(int64_t)k * 4];  // 32 bf16 per k-tile = four pieces
    }
  };
  auto store_x = [&](const u32x4 (&xb)[NXL], int stage) {
#pragma unroll
    for (int i = 0; i < NXL; ++i)
      if (wave + NWV * i < NPIECE) xs[stage][xkt[i]][xgrp[i]][lane] = xb[i];
  };

  f32x16 acc[CG][MT];
#pragma unroll
  for (int cg = 0; cg < CG; ++cg)
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[cg][t][r] = 0.f;

  // One chunk: for each 16-wide half of each k-tile, the MT activation
  // fragments (32 rows x 16 k each) come from LDS and meet the weight
  // fragments of the wave.  The fragments of the next half are requested before
  // the multiplies of the current one; the scheduling barriers pin that order
  // (left alone, the compiler moves each LDS read next to its first use and
  // every pair of multiplies waits for a full LDS round trip).
  // They are fetched in groups of BT row tiles (eight tiles at a time would need
  // 32 registers twice over); group g covers half h = g / NG, tiles (g % NG) BT ...
  constexpr int BT = MT == 8 ? 4 : MT;
  constexpr int NG = MT / BT;
  static_assert(NG * BT == MT, "row tiles must divide into groups");
  auto read_b = [&](bf16x8 (&b)[BT], int stage, int g) {
    const int h = g / NG, t0 = (g % NG) * BT;
    const int kt = h >> 1, kh = h & 1;
    const int r = l32 & 15;
    const int c = hi + 2 * kh;
#pragma unroll
    for (int t = 0; t < BT; ++t)
      b[t] = __builtin_bit_cast(bf16x8, xs[stage][kt][2 * (t0 + t) + (l32 >> 4)][4 * r + (c ^ ((r >> 2) & 3))]);
  };
  // One chunk of multiplies (the activation fragments of group g+1 are requested from LDS
  // before the multiplies of group g; the scheduling barriers pin that order).
  auto compute = [&](const u32x4 (&a)[CG][KC][2], int chunk, int stage) {
    bf16x8 b[2][BT];
    read_b(b[0], stage, 0);
#pragma unroll
    for (int g = 0; g < 2 * KC * NG; ++g) {
      const int h = g / NG, t0 = (g % NG) * BT;
      const int kt = h >> 1, kh = h & 1;
      if (g + 1 < 2 * KC * NG) read_b(b[(g + 1) & 1], stage, g + 1);
      __builtin_amdgcn_sched_barrier(0);
      const bool live = chunk * KC + kt < kt_end;
#pragma unroll
      for (int cg = 0; cg < CG; ++cg) {
        u32x4 w = a[cg][kt][kh];
        if (!live) w = u32x4{0u, 0u, 0u, 0u};
        const bf16x8 wv = __builtin_bit_cast(bf16x8, w);
#pragma unroll
        for (int t = 0; t < BT; ++t)
          acc[cg][t0 + t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, b[g & 1][t], acc[cg][t0 + t], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Software pipeline over k-chunks: weights through a ring of RING register buffers,
  // activations through two register buffers and two LDS stages; chunk c is multiplied
  // out of LDS stage c % 2 while chunk c+1 is written to the other stage, which every
  // wave finished reading before the barrier that ended step c-1.
  //
  // The eight waves of a workgroup leave that barrier together and share one address unit,
  // which takes ~25 cycles per 1 KiB load (measured: busy 1390 cycles per step of 56 loads,
  // against 1280 cycles of matrix work per SIMD and 2760 cycles per step), and a wave issues
  // in order: while all eight request their loads nobody multiplies.  So half of the waves
  // may run out of phase with the other half: they multiply first and request afterwards.
  //   early waves, step c: request activations c+2 and weights c+RING-1 (into the buffers
  //     freed in step c-1), multiply chunk c, write activations c+1 to LDS, barrier.
  //   late waves, step c: multiply chunk c, write activations c+1 to LDS, request
  //     activations c+3 and weights c+RING into the buffers just freed, barrier.
  // In both, the activations a step requests are older than its weights, so the wait that
  // precedes the LDS write (for a buffer requested two steps before it is written) never
  // covers the weight loads issued since.  The workgroup barrier is the bare instruction
  // (a __syncthreads would also wait for every outstanding load); the explicit wait before
  // it completes this wave's LDS writes and reads.  Both paths pass the same barriers.
  u32x4 ring[RING][CG][KC][2];
  u32x4 xb[2][NXL];
  auto run_early = [&]() {
    auto step = [&](const u32x4 (&cur)[CG][KC][2], u32x4 (&refill)[CG][KC][2], u32x4 (&xnew)[NXL],
                    const u32x4 (&xnext)[NXL], int chunk) {
      load_x(xnew, chunk + 2);
      __builtin_amdgcn_sched_barrier(0);
      load_w(refill, chunk + RING - 1);
      __builtin_amdgcn_sched_barrier(0);
      compute(cur, chunk, (chunk - chunk_begin) & 1);
      store_x(xnext, (chunk - chunk_begin + 1) & 1);
      FLY_WAIT_LGKMCNT0();
      FLY_BARE_BARRIER();
    };
    load_x(xb[0], chunk_begin);
    load_x(xb[1], chunk_begin + 1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int r = 0; r < RING - 1; ++r) load_w(ring[r], chunk_begin + r);
    store_x(xb[0], 0);
    FLY_WAIT_LGKMCNT0();
    FLY_BARE_BARRIER();
    // step r of a round of RING steps (RING even) refills register buffer r % 2
    int c = chunk_begin;
    while (c + RING <= chunk_end) {
#pragma unroll
      for (int r = 0; r < RING; ++r) step(ring[r], ring[(r + RING - 1) % RING], xb[r & 1], xb[(r + 1) & 1], c + r);
      c += RING;
    }
#pragma unroll
    for (int r = 0; r < RING - 1; ++r)
      if (c + r < chunk_end) step(ring[r], ring[(r + RING - 1) % RING], xb[r & 1], xb[(r + 1) & 1], c + r);
  };
  auto run_late = [&]() {
    auto step = [&](u32x4 (&cur)[CG][KC][2], u32x4 (&xnext)[NXL], int chunk) {
      compute(cur, chunk, (chunk - chunk_begin) & 1);
      store_x(xnext, (chunk - chunk_begin + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      load_x(xnext, chunk + 3);
      __builtin_amdgcn_sched_barrier(0);
      load_w(cur, chunk + RING);
      __builtin_amdgcn_sched_barrier(0);
      FLY_WAIT_LGKMCNT0();
      FLY_BARE_BARRIER();
    };
    load_x(xb[0], chunk_begin);
    load_x(xb[1], chunk_begin + 1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int r = 0; r < RING; ++r) load_w(ring[r], chunk_begin + r);
    store_x(xb[0], 0);
    __builtin_amdgcn_sched_barrier(0);
    load_x(xb[0], chunk_begin + 2);
    __builtin_amdgcn_sched_barrier(0);
    FLY_WAIT_LGKMCNT0();
    FLY_BARE_BARRIER();
    int c = chunk_begin;
    while (c + RING <= chunk_end) {
#pragma unroll
      for (int r = 0; r < RING; ++r) step(ring[r], xb[(r + 1) & 1], c + r);
      c += RING;
    }
#pragma unroll
    for (int r = 0; r < RING - 1; ++r)
      if (c + r < chunk_end) step(ring[r], xb[(r + 1) & 1], c + r);
  };
  // Half of the waves run late (phase 1).  Measured at the 405B width, gate/up GEMM, same box:
  // 136 rows 744 -> 702 us, 102 rows 641 -> 606, 170 rows 835 -> 797, 238 rows 1004 -> 965; at
  // 85 rows (three row tiles, where the weight stream alone sets the time) 580 -> 597, so the
  // launcher keeps every wave early there.  Which half is late makes no difference (waves
  // w < 4 or odd w: 702 and 703 us).
  if (chunk_begin < chunk_end) {
    if (phase == 1 && wave < NWV / 2)
      run_late();
    else
      run_early();
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
      for (int cg = 0; cg < CG; ++cg) {
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
      for (int cg = 0; cg < CG; ++cg) {
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
  } else {  // EPI_LMHEAD / EPI_LMSAMPLE: softmax statistics of this wave's 32 CG columns per row
    f32x4* o = (f32x4*)out;
    const int nparts = nblocks * NWV;
    const int part = nblock * NWV + wave;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int m = t * 32 + l32;
      const float sc = (row_scale != nullptr && m < M) ? row_scale[m] : 1.f;
      RowStat st = stat_empty();
#pragma unroll
      for (int cg = 0; cg < CG; ++cg) stat_update_tile32(st, acc[cg][t], sc, n0 + 32 * cg, hi, N);
      st = stat_merge(st, stat_shfl_xor(st, 32));
      if (hi == 0 && m < M) {
        f32x4 w;
        w.x = st.m;
        w.y = st.s;
        w.z = st.t;
        w.w = __int_as_float(st.idx);
        o[(int64_t)m * nparts + part] = w;
      }
      if constexpr (EPI == EPI_LMSAMPLE) {
        RowPick pk = pick_empty();
#pragma unroll
        for (int cg = 0; cg < CG; ++cg) pick_update_tile32(pk, acc[cg][t], sc, n0 + 32 * cg, hi, N, m, smp);
        pk = pick_merge(pk, pick_shfl_xor(pk, 32));
        if (hi == 0 && m < M) pick_store(smp, (int64_t)m * nparts + part, pk);
      }
    }
  }
}

template <int MT, int RING, int NWV, int CG>
static hipError_t launch_wide_mt(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale, int M,
                                 int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st,
                                 const LmSample& smp) {
  constexpr int WGS = 2 * CG * NWV;
  const int nblocks = (N / 16 + WGS - 1) / WGS;
  const int nchunks = (Kd / 32 + WIDE_KC - 1) / WIDE_KC;
  const int cps = (nchunks + plan.splits - 1) / plan.splits;
  dim3 grid(nblocks, plan.splits, 1), block(64 * NWV);
  const u32x4* W4 = (const u32x4*)Wp;
  const int knob = g_wide_phase.load();
  const int phase = knob == 0 ? (MT >= 4 ? 1 : 2) : knob;
  if (epi == EPI_PARTIAL)
    hipLaunchKernelGGL((gemm_bf16_wide_kernel<MT, EPI_PARTIAL, RING, NWV, CG>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks, phase, smp);
  else if (epi == EPI_SWIGLU)
    hipLaunchKernelGGL((gemm_bf16_wide_kernel<MT, EPI_SWIGLU, RING, NWV, CG>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks, phase, smp);
  else if (epi == EPI_LMHEAD)
    hipLaunchKernelGGL((gemm_bf16_wide_kernel<MT, EPI_LMHEAD, RING, NWV, CG>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks, phase, smp);
  else
    hipLaunchKernelGGL((gemm_bf16_wide_kernel<MT, EPI_LMSAMPLE, RING, NWV, CG>), grid, block, 0, st, X, W4, out,
                       row_scale, M, N, Kd, cps, nblocks, phase, smp);
  return hipGetLastError();
}

// plan.wide = number of 32-row tiles (3, 4, 5, 6 or 8).
hipError_t launch_gemm_bf16_wide(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale, int M,
                                 int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st,
                                 const LmSample& smp) {
  // Host-side shape checks: whole 16-column tiles and 32-row k-tiles, all rows
  // inside the one row block, every split owning at least one chunk.
  if (N % 16 != 0 || Kd % 32 != 0 || M < 1 || M > plan.wide * 32) return hipErrorInvalidValue;
  if (epi < EPI_PARTIAL || epi > EPI_LMSAMPLE) return hipErrorInvalidValue;
  if (epi == EPI_LMSAMPLE && smp.pick == nullptr) return hipErrorInvalidValue;
  if (plan.splits < 1 || (epi != EPI_PARTIAL && plan.splits != 1)) return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU && N % 32 != 0) return hipErrorInvalidValue;
  const int nchunks = (Kd / 32 + WIDE_KC - 1) / WIDE_KC;
  const int cps = (nchunks + plan.splits - 1) / plan.splits;
  if ((plan.splits - 1) * cps >= nchunks) return hipErrorInvalidValue;
  switch (plan.wide) {
    case 3: return launch_wide_mt<3, 6, WIDE_NWV, WIDE_CG>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 4: return launch_wide_mt<4, 6, WIDE_NWV, WIDE_CG>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 5: return launch_wide_mt<5, 4, WIDE_NWV, WIDE_CG>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 6: return launch_wide_mt<6, 4, WIDE_NWV, WIDE_CG>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 8: return launch_wide_mt<8, 2, WIDE_NWV, WIDE_CG>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
  }
  return hipErrorInvalidValue;
}

int gemm_bf16_wide_lmhead_parts(int N) { return (N + WIDE_COLS - 1) / WIDE_COLS * WIDE_NWV; }
int gemm_bf16_wide_cols() { return WIDE_COLS; }
