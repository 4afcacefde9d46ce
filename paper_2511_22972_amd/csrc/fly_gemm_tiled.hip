// LDS-tiled bf16 GEMM for large row counts (paper Sec. 2.1, Algorithm 1 step 2:
// the layer projections and the LM head of the verification forward when many
// sequences are verified together).
//
// With hundreds of activation rows the GEMMs stop being bound by streaming the
// weights and become dense contractions, so both operands are staged in LDS and
// every byte read from L2 is used by all waves of the workgroup.  The waves of
// a workgroup form a WGN x WGM grid; each wave owns 128 weight columns x 32 WM
// activation rows of out^T as 4 x WM tiles of v_mfma_f32_32x32x16_bf16 (weights
// = A operand, activations = B operand), so a workgroup covers 128 WGN columns
// x 32 WM WGM rows.  Global memory is copied straight into LDS by the LDS-direct
// loads (no staging registers) into a ring of NS k-steps of 32, with one
// barrier per k-step.
#include <type_traits>

#include "fly_common.h"

std::atomic<int> g_tiled_phase{0};  // tuning knob: 0 automatic, 1 half of the waves request mid-step, 2 every wave first

namespace {

__device__ __forceinline__ float silu_t(float x) { return x / (1.f + __expf(-x)); }

// One k-step (32 wide) of a workgroup tile in LDS:
//   w[strip][lane]  8 WGN packed weight tiles of 1 KiB exactly as in global memory
//   x[group][pos]   activation rows in groups of 16; a row is 64 bytes = four
//                   16-byte chunks, chunk c of row r stored at position
//                   4 r + (c ^ ((r >> 2) & 3)).  A 128-bit LDS read serves sixteen
//                   lanes per cycle (256 bytes, 64 banks) -- lanes 0-7 together with
//                   24-31, 8-15 with 16-23, the same in the upper half-wave
//                   (measured) --, and with this swizzle the sixteen rows such a
//                   set reads (rows 0-7 of one group, 8-15 of the next) fall into
//                   sixteen distinct 16-byte phases.
template <int WGN, int WGM, int WM>
struct TiledStage {
  u32x4 w[8 * WGN][64];
  u32x4 x[2 * WM * WGM][64];
};

// Operand fragments of one 16-wide half (kh) of a k-step: four weight tiles and
// WM activation tiles.
template <int WM>
struct TiledFrags {
  bf16x8 w[4], x[WM];
};

template <int WGN, int WGM, int WM>
__device__ __forceinline__ void tiled_read_frags(const TiledStage<WGN, WGM, WM>* st, TiledFrags<WM>& f,
                                                 int kh, int wn, int wm, int lane) {
  const int l32 = lane & 31, hi = lane >> 5;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    f.w[i] = __builtin_bit_cast(bf16x8, st->w[wn * 8 + 2 * i + (l32 >> 4)][(lane & 15) + 16 * (hi + 2 * kh)]);
#pragma unroll
  for (int t = 0; t < WM; ++t) {
    const int r = l32 & 15;
    const int c = hi + 2 * kh;
    f.x[t] = __builtin_bit_cast(bf16x8, st->x[(wm * WM + t) * 2 + (l32 >> 4)][4 * r + (c ^ ((r >> 2) & 3))]);
  }
}

template <int WM>
__device__ __forceinline__ void tiled_mma(const TiledFrags<WM>& f, f32x16 (&acc)[4][WM]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int t = 0; t < WM; ++t)
      acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.w[i], f.x[t], acc[i][t], 0, 0, 0);
}

}  // namespace

template <int WGN, int WGM, int WM, int EPI, int NS>
__global__ __launch_bounds__(WGN* WGM * 64) void gemm_bf16_tiled_kernel(
    const bf16_t* __restrict__ X, const u32x4* __restrict__ Wp, void* __restrict__ out,
    const float* __restrict__ row_scale, int M, int N, int Kd, int kt_per_split, int nblocks,
    int mblocks, int phase, LmSample smp) {
  constexpr int NW = WGN * WGM;                // waves
  constexpr int WLOADS = 8 * WGN / NW;         // LDS-direct loads per wave and stage: weights
  constexpr int XLOADS = 2 * WM * WGM / NW;    //                                      activations
  constexpr int LPW = WLOADS + XLOADS;
  constexpr int BM = 32 * WM * WGM;            // rows per workgroup
  static_assert(WLOADS * NW == 8 * WGN && XLOADS * NW == 2 * WM * WGM, "loads must divide evenly");
  static_assert(NS >= 3, "ring of at least three stages");
  // Workgroup -> (column block, row block): row blocks of one column block take
  // consecutive slots of one XCD so that they share the weight tiles in its L2.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int mblock = slot % mblocks;
  const int nblock = (slot / mblocks) * 8 + xcd;
  if (nblock >= nblocks) return;

  __shared__ TiledStage<WGN, WGM, WM> ring[NS];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wn = wave % WGN, wm = wave / WGN;
  const int ktiles = Kd / 32;
  const int nstrips = N / 16;
  const int kt_begin = blockIdx.y * kt_per_split;
  const int kt_end = min(kt_begin + kt_per_split, ktiles);
  const int nst = kt_end - kt_begin;
  const int kt_last = kt_end - 1;
  const int mrow0 = mblock * BM;

  // Global sources of this wave's share of a stage (k-tile 0).  Strips past the
  // end and rows past M are clamped to the last valid one (loaded, never stored).
  const u32x4* wsrc[WLOADS];
#pragma unroll
  for (int j = 0; j < WLOADS; ++j) {
    int strip = min(nblock * (8 * WGN) + wave * WLOADS + j, nstrips - 1);
    wsrc[j] = Wp + ((int64_t)strip * ktiles) * 64 + lane;
  }
  const bf16_t* xsrc[XLOADS];
#pragma unroll
  for (int j = 0; j < XLOADS; ++j) {
    const int r = lane >> 2;
    const int chunk = (lane & 3) ^ ((r >> 2) & 3);
    int row = min(mrow0 + (wave * XLOADS + j) * 16 + r, M - 1);
    xsrc[j] = X + (int64_t)row * Kd + chunk * 8;
  }
  auto issue_loads = [&](int s, int kt) {
    kt = min(kt, kt_last);  // surplus stages re-load the last one (never read)
#pragma unroll
    for (int j = 0; j < WLOADS; ++j)
      FLY_GLOBAL_TO_LDS16(wsrc[j] + (int64_t)kt * 64, &ring[s].w[wave * WLOADS + j][0]);
#pragma unroll
    for (int j = 0; j < XLOADS; ++j)
      FLY_GLOBAL_TO_LDS16(xsrc[j] + (int64_t)kt * 32, &ring[s].x[wave * XLOADS + j][0]);
  };

  f32x16 acc[4][WM];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int t = 0; t < WM; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][t][r] = 0.f;

#pragma unroll
  for (int s = 0; s < NS - 1; ++s) issue_loads(s, kt_begin + s);

  // Step c: wait for this wave's loads of stage c (the NS-2 younger stages may
  // still be in flight); barrier (everyone's loads of stage c have landed and
  // everyone is done reading stage c-1); refill the slot of stage c-1 with
  // stage c+NS-1; multiply stage c.  The eight waves leave the barrier together and
  // share one address unit (~25 cycles per 1 KiB load, 40 loads per step), and a wave
  // issues in order: a wave that requests first multiplies only once its loads are
  // accepted.  Half of the waves (LATE) therefore request their share between the two
  // halves of the step's multiplies; the slot they refill is free for the whole step,
  // and the number of younger loads at the wait is the same.
  auto steps = [&](auto late_c) {
    constexpr bool LATE = decltype(late_c)::value;
    int cur = 0, refill = NS - 1;
    for (int c = 0; c < nst; ++c) {
      FLY_WAIT_VMCNT((NS - 2) * LPW);
      FLY_BARE_BARRIER();
      if constexpr (!LATE) issue_loads(refill, kt_begin + c + NS - 1);
      TiledFrags<WM> f;
      tiled_read_frags<WGN, WGM, WM>(&ring[cur], f, 0, wn, wm, lane);
      tiled_mma<WM>(f, acc);
      if constexpr (LATE) issue_loads(refill, kt_begin + c + NS - 1);
      tiled_read_frags<WGN, WGM, WM>(&ring[cur], f, 1, wn, wm, lane);
      tiled_mma<WM>(f, acc);
      FLY_WAIT_LGKMCNT0();
      __builtin_amdgcn_sched_barrier(0);
      refill = cur;
      cur = cur + 1 == NS ? 0 : cur + 1;
    }
  };
  // Measured on the 1088 x 8192 x 128256 LM head, same box: every wave first 2140-2180 us, odd
  // waves late 2045-2070; the upper half of the waves late 2092, late after a quarter or three
  // quarters of the multiplies 2051-2073, four groups of waves at the four quarters 2136-2145.
  if (phase == 1 && (wave & 1))
    steps(std::true_type{});
  else
    steps(std::false_type{});
  FLY_WAIT_VMCNT(0);  // surplus (clamped) loads must have landed before the wave may end

  // ---- epilogues.  Accumulator register r of tile (i, t) in lane l is
  // out^T[n = n0 + 32 i + 8 (r/4) + 4 (l/32) + r%4][m = m0 + 32 t + l%32].
  const int l32 = lane & 31, hi = lane >> 5;
  const int n0 = (nblock * (8 * WGN) + wn * 8) * 16;
  const int m0 = mrow0 + wm * WM * 32;
  if constexpr (EPI == EPI_PARTIAL) {
    float* o = (float*)out + (int64_t)blockIdx.y * M * N;
#pragma unroll
    for (int t = 0; t < WM; ++t) {
      const int m = m0 + t * 32 + l32;
      if (m >= M) continue;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + 32 * i + 8 * q + 4 * hi;
          if (n < N) {
            f32x4 v = {acc[i][t][4 * q], acc[i][t][4 * q + 1], acc[i][t][4 * q + 2], acc[i][t][4 * q + 3]};
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
    for (int t = 0; t < WM; ++t) {
      const int m = m0 + t * 32 + l32;
      if (m >= M) continue;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (n0 + 32 * i + 31 >= N) continue;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          float a0 = silu_t(acc[i][t][4 * q + 0]) * acc[i][t][4 * q + 8];
          float a1 = silu_t(acc[i][t][4 * q + 1]) * acc[i][t][4 * q + 9];
          float a2 = silu_t(acc[i][t][4 * q + 2]) * acc[i][t][4 * q + 10];
          float a3 = silu_t(acc[i][t][4 * q + 3]) * acc[i][t][4 * q + 11];
          u32x2 pk;
          pk.x = pack_bf2(a0, a1);
          pk.y = pack_bf2(a2, a3);
          *(u32x2*)(o + (int64_t)m * Nh + (n0 + 32 * i) / 2 + 8 * q + 4 * hi) = pk;
        }
      }
    }
  } else {  // EPI_LMHEAD / EPI_LMSAMPLE: softmax statistics of this wave's 128 columns per row
    f32x4* o = (f32x4*)out;
    const int nparts = nblocks * WGN;
    const int part = nblock * WGN + wn;
#pragma unroll
    for (int t = 0; t < WM; ++t) {
      const int m = m0 + t * 32 + l32;
      const float sc = (row_scale != nullptr && m < M) ? row_scale[m] : 1.f;
      RowStat st = stat_empty();
#pragma unroll
      for (int i = 0; i < 4; ++i) stat_update_tile32(st, acc[i][t], sc, n0 + 32 * i, hi, N);
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
        for (int i = 0; i < 4; ++i) pick_update_tile32(pk, acc[i][t], sc, n0 + 32 * i, hi, N, m, smp);
        pk = pick_merge(pk, pick_shfl_xor(pk, 32));
        if (hi == 0 && m < M) pick_store(smp, (int64_t)m * nparts + part, pk);
      }
    }
  }
}

template <int WGN, int WGM, int WM>
static hipError_t launch_tiled_shape(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale,
                                     int M, int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st,
                                     const LmSample& smp) {
  constexpr int STAGE_KIB = 8 * WGN + 2 * WM * WGM;   // one k-step of the workgroup tile
  constexpr int NS = 4 * STAGE_KIB <= 144 ? 4 : 3;      // ring depth that fits the 160 KiB of LDS
  const int nblocks = (N / 16 + 8 * WGN - 1) / (8 * WGN);
  const int ktiles = Kd / 32;
  const int kps = (ktiles + plan.splits - 1) / plan.splits;
  if (plan.mblocks * (32 * WM * WGM) < M) return hipErrorInvalidValue;
  dim3 grid((nblocks + 7) / 8 * 8 * plan.mblocks, plan.splits, 1), block(WGN * WGM * 64);
  const u32x4* W4 = (const u32x4*)Wp;
  const int knob = g_tiled_phase.load();
  const int phase = knob == 0 ? 1 : knob;
  if (epi == EPI_PARTIAL)
    hipLaunchKernelGGL((gemm_bf16_tiled_kernel<WGN, WGM, WM, EPI_PARTIAL, NS>), grid, block, 0, st, X, W4,
                       out, row_scale, M, N, Kd, kps, nblocks, plan.mblocks, phase, smp);
  else if (epi == EPI_SWIGLU)
    hipLaunchKernelGGL((gemm_bf16_tiled_kernel<WGN, WGM, WM, EPI_SWIGLU, NS>), grid, block, 0, st, X, W4,
                       out, row_scale, M, N, Kd, kps, nblocks, plan.mblocks, phase, smp);
  else if (epi == EPI_LMHEAD)
    hipLaunchKernelGGL((gemm_bf16_tiled_kernel<WGN, WGM, WM, EPI_LMHEAD, NS>), grid, block, 0, st, X, W4,
                       out, row_scale, M, N, Kd, kps, nblocks, plan.mblocks, phase, smp);
  else
    hipLaunchKernelGGL((gemm_bf16_tiled_kernel<WGN, WGM, WM, EPI_LMSAMPLE, NS>), grid, block, 0, st, X, W4,
                       out, row_scale, M, N, Kd, kps, nblocks, plan.mblocks, phase, smp);
  return hipGetLastError();
}

// plan.tiled selects the workgroup shape, see tiled_shape_rows().
hipError_t launch_gemm_bf16_tiled(const bf16_t* X, const bf16_t* Wp, void* out, const float* row_scale,
                                  int M, int N, int Kd, const GemmPlan& plan, int epi, hipStream_t st,
                                  const LmSample& smp) {
  if (N % 16 != 0 || Kd % 32 != 0 || M < 1) return hipErrorInvalidValue;
  if (epi < EPI_PARTIAL || epi > EPI_LMSAMPLE) return hipErrorInvalidValue;
  if (epi == EPI_LMSAMPLE && smp.pick == nullptr) return hipErrorInvalidValue;
  if (plan.splits < 1 || (epi != EPI_PARTIAL && plan.splits != 1)) return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU && (N % 32 != 0)) return hipErrorInvalidValue;
  // every split must own at least one k-tile (the kernel's prologue assumes it)
  const int ktiles = Kd / 32;
  const int kps = (ktiles + plan.splits - 1) / plan.splits;
  if ((plan.splits - 1) * kps >= ktiles) return hipErrorInvalidValue;
  switch (plan.tiled) {
    case 2: return launch_tiled_shape<2, 2, 2>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 3: return launch_tiled_shape<2, 2, 3>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 4: return launch_tiled_shape<2, 4, 2>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
    case 6: return launch_tiled_shape<2, 4, 3>(X, Wp, out, row_scale, M, N, Kd, plan, epi, st, smp);
  }
  return hipErrorInvalidValue;
}

// Rows and columns a workgroup of shape `tiled` covers (0 if the shape does not exist).
int gemm_bf16_tiled_rows(int tiled) {
  return tiled == 2 ? 128 : tiled == 3 ? 192 : tiled == 4 ? 256 : tiled == 6 ? 384 : 0;
}
int gemm_bf16_tiled_cols(int tiled) { return gemm_bf16_tiled_rows(tiled) ? 256 : 0; }

int gemm_bf16_tiled_lmhead_parts(int N, int tiled) {
  const int cols = gemm_bf16_tiled_cols(tiled);
  return cols ? (N + cols - 1) / cols * (cols / 128) : 0;
}
