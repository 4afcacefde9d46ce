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
// A workgroup of eight waves streams 64-key stages through an LDS ring filled
// by LDS-direct loads.  With up to four 32-row query tiles (KS = 2) wave w owns
// tile w/2 and the keys 32 (w%2) .. +31 of every stage, so that few rows still
// spread over all four SIMDs; the two key halves of a tile are merged through
// LDS at the end.  With five to eight tiles (KS = 1) wave w owns tile w and all
// 64 keys of a stage.  More than 256 rows are divided over several query blocks
// (workgroups) that stream the same keys.
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
#define ATT_STAGE_BYTES (ATT_KC * ATT_KROW + ATT_HD * ATT_VROW)  // 32 KiB
#define ATT_NWAVES 8
#define ATT_NSTG 4                      // stages in the LDS ring (128 KiB); three are in flight
// Rows are stored unpadded; the 16-byte pieces of a row are permuted so that
// the operand-order loads are free of bank conflicts.  A 128-bit LDS read serves
// sixteen lanes per cycle (256 bytes, 64 banks): lanes 0-7 together with 24-31,
// 8-15 with 16-23, and the same in the upper half-wave (measured).  Key rows
// (256 bytes) XOR the piece index with the low four bits of the key, bit 2
// flipped when bit 3 is set: the sixteen keys such a lane set reads (see
// ATT_KPERM) then take sixteen distinct pieces.  V^T rows (128 bytes, so the row's
// parity is the top bit of the phase) XOR it with (row & 7), bit 0 flipped for rows
// 16-31 of a 32-row tile: rows 0-7 and 24-31, and 8-15 and 16-23, never meet.
#define ATT_KSWZ(key, piece) (((piece) ^ (((key) & 15) ^ ((((key) >> 3) & 1) << 2))) * 16)
#define ATT_VSWZ(row, piece) (((piece) ^ (((row) & 7) ^ (((row) >> 4) & 1))) * 16)
// Row i of a 32-key score tile holds key ATT_KPERM(i) of the tile (bits 2 and 3
// of i swapped).  With this order the sixteen scores a lane holds of one query
// row are two runs of eight consecutive keys, i.e. exactly the operand order
// of the P V product, whose V^T fragments are then whole 16-byte pieces.
#define ATT_KPERM(i) (((i) & 0x13) | (((i) & 4) << 1) | (((i) & 8) >> 1))

// LDS-direct load: every lane gives its own global address of 16 bytes, the wave's
// 1 KiB lands at lds_base + 16 * lane (lds_base wave-uniform, passed in M0).
// Issued from inline assembly so that the compiler's automatic wait insertion,
// which cannot tell the ring slots apart, does not wait for ALL outstanding
// loads before every LDS read; the waits for these loads are placed by hand.
// Unknown to the compiler's counters, they can only make its own vmcnt waits
// longer than needed, never shorter.  The hand-counted waits rely on LDS-direct
// loads completing in issue order among themselves; no register load is in
// flight while they count (the query loads are waited for first).  M0 is reserved
// by the compiler, which warns about the clobber; nothing else here uses M0.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void att_global_to_lds16(const void* gptr, const void* lds_base) {
  const uint32_t lds_addr =
      (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)lds_base;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(lds_addr), "v"(gptr)
               : "memory", "m0");
}
#pragma clang diagnostic pop
// s_waitcnt vmcnt(n) only / lgkmcnt(0) only.
#define ATT_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)
#define ATT_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(0xC07F)
// Workgroup barrier without the fence of __syncthreads (which would wait for
// all outstanding LDS-direct loads, also those of the stages being prefetched).
#define ATT_BARE_BARRIER()              \
  asm volatile("" ::: "memory");        \
  __builtin_amdgcn_sched_barrier(0);    \
  __builtin_amdgcn_s_barrier();         \
  __builtin_amdgcn_sched_barrier(0);    \
  asm volatile("" ::: "memory")

std::atomic<int> g_attn_force_splits{0};  // tuning knobs (0 = automatic)
std::atomic<int> g_attn_force_block_tiles{0};
std::atomic<int> g_attn_phase{0};  // 0 automatic, 1 odd waves late, 2 every wave first

AttnPlan plan_attention(int B, int K, int Hq, int Hkv, int max_total_len) {
  AttnPlan p;
  int G = Hq / Hkv;
  int R = G * (K + 1);
  int qt = (R + 31) / 32;  // 32-row query tiles
  // A workgroup holds up to eight tiles; more rows are divided evenly over
  // several query blocks.  Up to four tiles take the key-split kernel.
  int per_block = g_attn_force_block_tiles ? g_attn_force_block_tiles.load() : 8;
  p.qblocks = (qt + per_block - 1) / per_block;
  p.block_tiles = (qt + p.qblocks - 1) / p.qblocks;
  int wgs = B * Hkv * p.qblocks;
  int chunks = (max_total_len + ATT_KC - 1) / ATT_KC;
  if (chunks < 1) chunks = 1;
  // one workgroup per compute unit (the LDS ring allows no more), at least two
  // stages per split; the splits fill the 256 units without spilling into a second,
  // nearly empty round of workgroups
  int want = g_attn_force_splits ? g_attn_force_splits.load() : (wgs >= 256 ? 1 : 256 / wgs);
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

// KS = 2: a wave owns (tile wave/2, key half wave%2); KS = 1: (tile wave, all keys).
template <int KS>
__global__ __launch_bounds__(ATT_NWAVES * 64) void attention_bf16_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kcache, const bf16_t* __restrict__ vcache,
    const int32_t* __restrict__ kv_len, float* __restrict__ ws, int K, int Hq, int Hkv, int capacity,
    int chunk_keys, int qblocks, int block_tiles, int nsplit, int npairs, float scale, int phase) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[ATT_NSTG * ATT_STAGE_BYTES];
  constexpr int NW = ATT_NWAVES;
  constexpr int nthreads = NW * 64;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: scalar branches
  const int h = lane >> 5, l32 = lane & 31;
  constexpr int NKT = 2 / KS;  // 32-key tiles of a stage this wave multiplies
  const int tile = KS == 2 ? wave >> 1 : wave;  // this wave's query tile
  const int half = KS == 2 ? wave & 1 : 0;      // and key half of a stage
  // Workgroup -> (query block, split, pair).  Workgroups are dealt to the eight
  // XCDs (each with its own L2) round-robin by linear id; the query blocks of one
  // (pair, split) stream the same keys, so they take consecutive slots of ONE
  // XCD: they run together and all but the first find the keys in that L2.
  const int xcd = blockIdx.x & 7, wslot = blockIdx.x >> 3;
  const int qb = wslot % qblocks;
  const int unit = (wslot / qblocks) * 8 + xcd;
  if (unit >= nsplit * npairs) return;  // padding of the last group of eight (uniform per workgroup)
  const int split = unit % nsplit, pair = unit / nsplit;
  const int b = pair / Hkv, kvh = pair % Hkv;
  const int G = Hq / Hkv;
  const int R = G * (K + 1);
  const int row_begin = qb * block_tiles * 32;  // this query block's rows
  const int row_end = min(R, row_begin + block_tiles * 32);
  const int L = kv_len[b];
  int total = L + K + 1;  // keys visible to the last query
  if (total > capacity) total = capacity;  // the host checks this bound; never read past the slab
  const int key_begin = split * chunk_keys;
  int key_end = key_begin + chunk_keys;
  if (key_end > total) key_end = total;

  const bf16_t* kbase = kcache + ((int64_t)b * Hkv + kvh) * (int64_t)capacity * ATT_HD;
  const bf16_t* vbase = vcache + ((int64_t)b * Hkv + kvh) * (int64_t)ATT_HD * capacity;

  const int nstages = key_end > key_begin ? (key_end - key_begin + ATT_KC - 1) / ATT_KC : 0;

  // ---- stage loads.  A stage is 32 wave-level LDS-direct loads of 1 KiB:
  // loads 0..15 bring four key rows each (lane: row l/16, 16-byte piece l%16),
  // loads 16..31 eight V^T rows each (lane: row l/8, piece l%8); the lane
  // fetches the piece that the swizzle assigns to its LDS position.  Wave w
  // issues loads w*LPW .. w*LPW+LPW-1.  A stage starts at a multiple of 64 below
  // key_end and the capacity is a multiple of 64, so every address is inside
  // the slab; keys at or past key_end hold whatever the allocation held, see
  // the tail fix-up below.
  constexpr int LPW = 32 / NW;
  const bf16_t* src[LPW];
#pragma unroll
  for (int j = 0; j < LPW; ++j) {
    const int ld = wave * LPW + j;
    if (ld < 16) {
      const int key = 4 * ld + (lane >> 4);
      src[j] = kbase + (int64_t)(key_begin + key) * ATT_HD + ATT_KSWZ(key, lane & 15) / 2;
    } else {
      const int row = 8 * (ld - 16) + (lane >> 3);
      src[j] = vbase + (int64_t)row * capacity + key_begin + ATT_VSWZ(row, lane & 7) / 2;
    }
  }
  auto issue_stage = [&](int slot, int stage_idx) {
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
      const int ld = wave * LPW + j;
      const int64_t adv = (ld < 16) ? (int64_t)stage_idx * ATT_KC * ATT_HD : (int64_t)stage_idx * ATT_KC;
      att_global_to_lds16(src[j] + adv, smem + slot * ATT_STAGE_BYTES + ld * 1024);
    }
  };

  // ---- this wave's query tile: operand B of S^T = K Q^T (32x32x16 tiles), lane
  // holds Q[row = row_begin + 32*tile + l32][hd = 16*kk + 8h .. +8].  The loads
  // are waited for before the first stage load is issued, so that the
  // hand-counted waits below see stage loads only.
  u32x4 qf[8];
  const int qr = row_begin + tile * 32 + l32;
  const bool row_ok = qr < row_end;
  const int qlimit = row_ok ? L + qr / G + 1 : 0;  // number of keys visible to this row
  {
    const int rc = row_ok ? qr : R - 1;  // clamp: the load is unconditional, the value is masked
    const int i = rc / G, gq = rc % G;
    const bf16_t* qp = q + ((int64_t)(b * (K + 1) + i) * Hq + kvh * G + gq) * ATT_HD;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      u32x4 v = *(const u32x4*)(qp + 16 * kk + 8 * h);
      qf[kk] = row_ok ? v : u32x4{0u, 0u, 0u, 0u};
    }
  }
  ATT_WAIT_VMCNT(0);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 0; s < ATT_NSTG - 1; ++s)
    if (s < nstages) issue_stage(s, s);

  f32x16 oacc[4];  // O^T[hd = 32*ht + 8*(r/4) + 4h + r%4][row l32], this wave's keys only
  float mrun = -INFINITY, lrun = 0.f;
#pragma unroll
  for (int ht = 0; ht < 4; ++ht)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[ht][r] = 0.f;

  // The wave's 32 keys of one stage (LDS buffer `stage`, first key kstart).
  //
  // Probabilities are formed relative to an INTEGER base-2 exponent n >= max s',
  // s' = (q.k) * log2(e)/sqrt(hd), n = ceil of the running maximum: when the
  // maximum grows, earlier terms are rescaled by an exact power of two, which
  // commutes with the bf16 rounding of P.  The result is the same as rounding
  // 2^(s' - n_final) once, independent of how the cache is chunked or split.
  const bool wave_has_rows = row_begin + tile * 32 < row_end;
  auto compute_stage = [&](int stage, int kstart) {
    if (!wave_has_rows) return;  // this wave only helps with the loads
    const unsigned char* kb = smem + stage * ATT_STAGE_BYTES;
    const unsigned char* vb = kb + ATT_KC * ATT_KROW;

    // S^T = K Q^T for the wave's key tiles; register r of tile kt in a lane is the
    // score of key kfirst + 32*kt + 16*(r/8) + 8h + r%8 (see ATT_KPERM) and query row l32.
    const int kfirst = kstart + half * 32;
    f32x16 sacc[NKT];
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[kt][r] = 0.f;
      const int key = (half + kt) * 32 + ATT_KPERM(l32);
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        u32x4 araw = *(const u32x4*)(kb + key * ATT_KROW + ATT_KSWZ(key, 2 * kk + h));
        sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, araw),
                                                           __builtin_bit_cast(bf16x8, qf[kk]), sacc[kt], 0, 0, 0);
      }
    }
    if (kfirst + 32 * NKT > L + 1) {  // keys below L+1 are visible to every row (wave-uniform branch)
#pragma unroll
      for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int key = kfirst + 32 * kt + 16 * (r >> 3) + 8 * h + (r & 7);
          if (key >= qlimit) sacc[kt][r] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
      for (int r = 0; r < 16; r += 4)
        mx = fmaxf(mx, fmaxf(fmaxf(sacc[kt][r], sacc[kt][r + 1]), fmaxf(sacc[kt][r + 2], sacc[kt][r + 3])));
    mx = fmaxf(mx, __shfl_xor(mx, 32, FLY_WAVE));
    const float mnew = fmaxf(mrun, ceilf(mx * scale));  // scale > 0: max commutes with it
    // rows with nothing visible yet keep n = -inf; avoid inf - inf
    const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
    if (__ballot(mnew != mrun) != 0ull) {  // wave-uniform: some row's exponent grew
      const float corr = fast_exp2(mrun - msafe);  // exact power of two (0 when mrun = -inf)
      lrun *= corr;
#pragma unroll
      for (int ht = 0; ht < 4; ++ht) oacc[ht] *= corr;
      mrun = mnew;
    }
    u32x4 pb[NKT][2];  // P as operand of the P V product: 16-key steps, 8 keys per lane each
    float lsum = 0.f;
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        float pv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) pv[e] = fast_exp2(fmaf(sacc[kt][8 * j + e], scale, -msafe));
        lsum += ((pv[0] + pv[1]) + (pv[2] + pv[3])) + ((pv[4] + pv[5]) + (pv[6] + pv[7]));
        pb[kt][j] = u32x4{pack_bf2_hw(pv[0], pv[1]), pack_bf2_hw(pv[2], pv[3]), pack_bf2_hw(pv[4], pv[5]),
                          pack_bf2_hw(pv[6], pv[7])};
      }
    lrun += lsum;

    // O^T += V^T P^T.  Step (kt, j) covers 16 keys; the lane's eight keys
    // 32*(half + kt) + 16j + 8h .. +7 are piece 4*(half + kt) + 2j + h of a V^T row.
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int ht = 0; ht < 4; ++ht) {
          const int vrow = ht * 32 + l32;
          u32x4 araw = *(const u32x4*)(vb + vrow * ATT_VROW + ATT_VSWZ(vrow, 4 * (half + kt) + 2 * j + h));
          oacc[ht] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, araw), __builtin_bit_cast(bf16x8, pb[kt][j]), oacc[ht], 0, 0, 0);
        }
      }
  };

  // Pipeline over the stages of this split.  Step c: wait for this wave's loads
  // of stage c (up to two younger stages stay in flight); barrier (everyone's
  // loads of stage c have landed, everyone is done reading stage c-1); refill
  // the slot of stage c-1 with stage c+3; multiply stage c out of LDS.
  const bool late = phase == 1 && (wave & 1);  // this wave requests its share of a stage after multiplying
  int slot = 0, refill = ATT_NSTG - 1;
  for (int c = 0; c < nstages; ++c) {
    const int younger = min(ATT_NSTG - 2, nstages - 1 - c);  // stages issued after stage c
    if (younger >= 2) ATT_WAIT_VMCNT(2 * LPW);
    else if (younger == 1) ATT_WAIT_VMCNT(LPW);
    else ATT_WAIT_VMCNT(0);
    ATT_BARE_BARRIER();
    if (!late && c + ATT_NSTG - 1 < nstages) issue_stage(refill, c + ATT_NSTG - 1);
    const int kstart = key_begin + c * ATT_KC;
    if (kstart + ATT_KC > key_end) {
      // Last stage of the cache: V^T columns of keys at or past key_end hold
      // whatever the allocation held (possibly NaN patterns, and 0 * NaN would
      // poison the sums): zero them in LDS.  Scores of such keys are replaced by
      // -inf above, so the key rows need no such care.  Workgroup-uniform branch.
      unsigned char* vb = smem + slot * ATT_STAGE_BYTES + ATT_KC * ATT_KROW;
      const int nvalid_stage = key_end - kstart;  // 1..63
      for (int item = tid; item < ATT_HD * 8; item += nthreads) {
        const int row = item >> 3, piece = item & 7;
        const int nvalid = nvalid_stage - piece * 8;  // valid keys in this 8-key piece
        if (nvalid < 8) {
          u32x4* pv = (u32x4*)(vb + row * ATT_VROW + ATT_VSWZ(row, piece));
          u32x4 v = *pv;
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            uint32_t keep = (2 * w < nvalid ? 0xFFFFu : 0u) | (2 * w + 1 < nvalid ? 0xFFFF0000u : 0u);
            v[w] &= keep;
          }
          *pv = v;
        }
      }
      __syncthreads();  // no younger stage loads are outstanding here
    }
    compute_stage(slot, kstart);
    if (late && c + ATT_NSTG - 1 < nstages) issue_stage(refill, c + ATT_NSTG - 1);
    ATT_WAIT_LGKMCNT0();
    __builtin_amdgcn_sched_barrier(0);
    refill = slot;
    slot = slot + 1 == ATT_NSTG ? 0 : slot + 1;
  }

  // ---- this split's partial: O [R, hd], n [R], l [R].  With split keys the two
  // halves of each tile are first merged through LDS (the ring is free now): the
  // odd wave hands over its O, n and l, the even wave combines them with its own
  // (n = max of the two integer exponents, both sides rescaled by exact powers
  // of two, the even half added first).
  lrun += __shfl_xor(lrun, 32, FLY_WAVE);
  float* xo = (float*)smem + tile * (16 * 4 * 64 + 64);  // [ht][r][lane] floats, then n[32], l[32]
  float w0 = 1.f, w1 = 0.f;
  if constexpr (KS == 2) {
    __syncthreads();  // all stage reads done (no stage loads are outstanding after the last step)
    if (half == 1 && wave_has_rows) {
#pragma unroll
      for (int ht = 0; ht < 4; ++ht)
#pragma unroll
        for (int r = 0; r < 16; ++r) xo[(ht * 16 + r) * 64 + lane] = oacc[ht][r];
      if (h == 0) {
        xo[16 * 4 * 64 + l32] = mrun;
        xo[16 * 4 * 64 + 32 + l32] = lrun;
      }
    }
    __syncthreads();
    if (half == 0 && wave_has_rows) {
      const float m1 = xo[16 * 4 * 64 + l32], l1 = xo[16 * 4 * 64 + 32 + l32];
      const float mm = fmaxf(mrun, m1);
      const float msafe = (mm == -INFINITY) ? 0.f : mm;
      w0 = fast_exp2(mrun - msafe);  // 0 for an empty half
      w1 = fast_exp2(m1 - msafe);
      lrun = lrun * w0 + l1 * w1;
      mrun = mm;
    }
  }
  if (half == 0 && row_ok) {
    float* obase = ws + ((int64_t)pair * nsplit + split) * (int64_t)R * (ATT_HD + 2);
    float* mbase = obase + (int64_t)R * ATT_HD;
    float* lbase = mbase + R;
#pragma unroll
    for (int ht = 0; ht < 4; ++ht)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = oacc[ht][4 * qd + e];
          if constexpr (KS == 2) v[e] = v[e] * w0 + xo[(ht * 16 + 4 * qd + e) * 64 + lane] * w1;
        }
        *(f32x4*)(obase + (int64_t)qr * ATT_HD + ht * 32 + 8 * qd + 4 * h) = v;
      }
    if (h == 0) {
      mbase[qr] = mrun;
      lbase[qr] = lrun;
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
#pragma unroll 8
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
#pragma unroll 8
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
  if (p.nsplit < 1 || p.nsplit > ATT_MAX_SPLITS) return hipErrorInvalidValue;
  if (p.qblocks < 1 || p.block_tiles < 1 || p.block_tiles > 8) return hipErrorInvalidValue;
  int G = Hq / Hkv, R = G * (K + 1);
  if (p.qblocks * p.block_tiles * 32 < R) return hipErrorInvalidValue;
  const int units = p.nsplit * B * Hkv;
  dim3 grid((units + 7) / 8 * 8 * p.qblocks), block(ATT_NWAVES * 64);
  float scale = (float)(1.4426950408889634 / sqrt((double)hd));  // log2(e) / sqrt(hd)
  const int knob = g_attn_phase.load();
  const int phase = knob == 0 ? 1 : knob;  // odd waves request their share of a stage after multiplying (1-1.5% faster)
  if (p.block_tiles <= 4)
    hipLaunchKernelGGL(attention_bf16_kernel<2>, grid, block, 0, st, q, kcache, vcache, kv_len, ws, K, Hq,
                       Hkv, capacity, p.chunk_keys, p.qblocks, p.block_tiles, p.nsplit, B * Hkv, scale, phase);
  else
    hipLaunchKernelGGL(attention_bf16_kernel<1>, grid, block, 0, st, q, kcache, vcache, kv_len, ws, K, Hq,
                       Hkv, capacity, p.chunk_keys, p.qblocks, p.block_tiles, p.nsplit, B * Hkv, scale, phase);
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
#pragma unroll 16
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
#pragma unroll 8
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
