// Drafting by prompt lookup and the bookkeeping of the decode loop
// (paper Sec. 2.3; Algorithm 1, outer loop and step 1; Eq. 12).
//
// Both kernels are integer-only and tiny next to the verification forward;
// they exist so that a whole multi-round decode runs on the device without a
// host round trip per round: draft -> verify -> roll forward.
#include "fly_common.h"

#define PLD_THREADS 256

// Prompt-lookup drafter (Sec. 2.3: n-gram retrieval over the context; the
// parameters are this library's): for the sequence y of length L, find the
// longest n <= n_max such that the last n tokens occur earlier, ending at some
// e < L, and among those occurrences the latest; propose the K tokens that
// follow it, continuing through the proposal itself where the copy runs past
// the end of y.  Without an occurrence the last token is repeated.
// Output: tokens[b] = (y[L-1], draft_1..draft_K), the block the verification
// step takes; ngram[b] = n (0: no occurrence).
// One workgroup per sequence: every thread scores end positions e by the
// length of the common suffix of y[0..e) and y (capped at n_max); the best
// (n, e) pair is reduced as a 64-bit key.
__global__ __launch_bounds__(PLD_THREADS) void pld_draft_kernel(const int32_t* __restrict__ ctx,
                                                                const int32_t* __restrict__ ctx_len,
                                                                int ctx_capacity, int K, int n_max,
                                                                int32_t* __restrict__ tokens,
                                                                int32_t* __restrict__ ngram) {
  __shared__ unsigned long long wbest[PLD_THREADS / 64];
  __shared__ unsigned long long best_all;
  const int b = blockIdx.x, tid = threadIdx.x;
  const int32_t* y = ctx + (int64_t)b * ctx_capacity;
  int L = ctx_len[b];
  if (L > ctx_capacity) L = ctx_capacity;  // the host checks the bound; never read past the row
  int32_t* out = tokens + (int64_t)b * (K + 1);
  if (L < 1) {  // no sequence: a block of zeros (the host rules this out)
    for (int i = tid; i <= K; i += PLD_THREADS) out[i] = 0;
    if (tid == 0 && ngram) ngram[b] = 0;
    return;
  }
  unsigned long long best = 0;
  for (int e = 1 + tid; e < L; e += PLD_THREADS) {
    int n = 0;
    const int cap = min(n_max, e);
    while (n < cap && y[e - 1 - n] == y[L - 1 - n]) ++n;
    if (n > 0) {
      unsigned long long key = ((unsigned long long)n << 32) | (unsigned)e;
      best = key > best ? key : best;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    unsigned lo = __shfl_xor((unsigned)best, o, FLY_WAVE);
    unsigned hi = __shfl_xor((unsigned)(best >> 32), o, FLY_WAVE);
    unsigned long long other = ((unsigned long long)hi << 32) | lo;
    best = other > best ? other : best;
  }
  if ((tid & 63) == 0) wbest[tid >> 6] = best;
  __syncthreads();
  if (tid == 0) {
    unsigned long long m = wbest[0];
#pragma unroll
    for (int w = 1; w < PLD_THREADS / 64; ++w) m = wbest[w] > m ? wbest[w] : m;
    best_all = m;
    const int n = (int)(m >> 32), e = (int)(m & 0xFFFFFFFFu);
    out[0] = y[L - 1];
    // the copy may overlap its own output: sequential, K <= 63
    for (int i = 0; i < K; ++i) {
      int32_t t;
      if (n == 0) t = y[L - 1];
      else t = (e + i < L) ? y[e + i] : out[1 + (e + i - L)];
      out[1 + i] = t;
    }
    if (ngram) ngram[b] = n;
  }
}

hipError_t launch_pld_draft(const int32_t* ctx, const int32_t* ctx_len, int ctx_capacity, int B, int K,
                            int n_max, int32_t* tokens, int32_t* ngram, hipStream_t st) {
  hipLaunchKernelGGL(pld_draft_kernel, dim3(B), dim3(PLD_THREADS), 0, st, ctx, ctx_len, ctx_capacity, K,
                     n_max, tokens, ngram);
  return hipGetLastError();
}

// End of a round (Algorithm 1: y <- concat[y, kept drafts, y_s]; s += j; t += 1):
// append the kept drafts and the correction / bonus token to the sequence, move
// the cache length to the rows that stay valid, accumulate the statistics.
// A sequence whose row is full stops growing (the host sizes the rows so that
// this does not happen).
__global__ void roll_forward_kernel(int32_t* __restrict__ ctx, int32_t* __restrict__ ctx_len,
                                    int32_t* __restrict__ kv_len, int ctx_capacity, int B, int K,
                                    const int32_t* __restrict__ tokens,
                                    const int32_t* __restrict__ accept_len,
                                    const int32_t* __restrict__ next_token,
                                    const int32_t* __restrict__ kv_len_out,
                                    const int32_t* __restrict__ n_loose,
                                    int64_t* __restrict__ accepted_total, int32_t* __restrict__ rounds_done,
                                    int64_t* __restrict__ loose_total, int32_t* __restrict__ trace_row) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int a = accept_len[b];
  const int s = a + 1;
  const int L = ctx_len[b];
  if (L + s > ctx_capacity) {
    if (trace_row) trace_row[b] = 0;
    return;
  }
  int32_t* y = ctx + (int64_t)b * ctx_capacity;
  const int32_t* blk = tokens + (int64_t)b * (K + 1);
  for (int i = 0; i < a; ++i) y[L + i] = blk[1 + i];
  y[L + a] = next_token[b];
  ctx_len[b] = L + s;
  kv_len[b] = kv_len_out[b];
  if (accepted_total) accepted_total[b] += s;
  if (rounds_done) rounds_done[b] += 1;
  if (loose_total && n_loose) loose_total[b] += n_loose[b];
  if (trace_row) trace_row[b] = s;
}

hipError_t launch_roll_forward(int32_t* ctx, int32_t* ctx_len, int32_t* kv_len, int ctx_capacity, int B,
                               int K, const int32_t* tokens, const int32_t* accept_len,
                               const int32_t* next_token, const int32_t* kv_len_out,
                               const int32_t* n_loose, int64_t* accepted_total, int32_t* rounds_done,
                               int64_t* loose_total, int32_t* trace_row, hipStream_t st) {
  hipLaunchKernelGGL(roll_forward_kernel, dim3((B + 63) / 64), dim3(64), 0, st, ctx, ctx_len, kv_len,
                     ctx_capacity, B, K, tokens, accept_len, next_token, kv_len_out, n_loose, accepted_total,
                     rounds_done, loose_total, trace_row);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Drafting with a draft model (Algorithm 1 step 1 with a model M_D): K greedy
// forward passes of the drafter per round.  These kernels only move token ids
// and cache lengths between the passes, so that the passes chain on the device.
//
// Sequence b has n = ctx_len[b] tokens; the drafter's cache holds valid rows for
// the positions before n-2 (the rows of the last two tokens are computed again
// every round: the last one is new, and the one before it is the only row that
// may be missing, namely after a round that kept all K drafts).  Pass 1 takes
// the two tokens ctx[n-2], ctx[n-1] against n-2 cached rows; pass i >= 2 takes
// draft i-1 against n+i-2 rows.
// ---------------------------------------------------------------------------
__global__ void draft_prepare_kernel(const int32_t* __restrict__ ctx, const int32_t* __restrict__ ctx_len,
                                     int ctx_capacity, int B, int K, int32_t* __restrict__ tok2,
                                     int32_t* __restrict__ len_steps) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int n = ctx_len[b];
  n = n < 2 ? 2 : (n > ctx_capacity ? ctx_capacity : n);  // the host rules both out; never read outside the row
  const int32_t* y = ctx + (int64_t)b * ctx_capacity;
  tok2[2 * b] = y[n - 2];
  tok2[2 * b + 1] = y[n - 1];
  len_steps[b] = n - 2;
  for (int j = 1; j < K; ++j) len_steps[(int64_t)j * B + b] = n + j - 1;
}

// drafts[0][b] = argmax of the second row of pass 1
__global__ void draft_pick_kernel(const int32_t* __restrict__ argmax2, int B, int32_t* __restrict__ first) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) first[b] = argmax2[2 * b + 1];
}

// tokens[b] = (y_{-1}, draft_1..draft_K), the block the verification step takes
__global__ void draft_assemble_kernel(const int32_t* __restrict__ tok2, const int32_t* __restrict__ drafts,
                                      int B, int K, int32_t* __restrict__ tokens) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int32_t* out = tokens + (int64_t)b * (K + 1);
  out[0] = tok2[2 * b + 1];
  for (int i = 0; i < K; ++i) out[1 + i] = drafts[(int64_t)i * B + b];
}

hipError_t launch_draft_prepare(const int32_t* ctx, const int32_t* ctx_len, int ctx_capacity, int B, int K,
                                int32_t* tok2, int32_t* len_steps, hipStream_t st) {
  hipLaunchKernelGGL(draft_prepare_kernel, dim3((B + 63) / 64), dim3(64), 0, st, ctx, ctx_len, ctx_capacity, B,
                     K, tok2, len_steps);
  return hipGetLastError();
}
hipError_t launch_draft_pick(const int32_t* argmax2, int B, int32_t* first, hipStream_t st) {
  hipLaunchKernelGGL(draft_pick_kernel, dim3((B + 63) / 64), dim3(64), 0, st, argmax2, B, first);
  return hipGetLastError();
}
hipError_t launch_draft_assemble(const int32_t* tok2, const int32_t* drafts, int B, int K, int32_t* tokens,
                                 hipStream_t st) {
  hipLaunchKernelGGL(draft_assemble_kernel, dim3((B + 63) / 64), dim3(64), 0, st, tok2, drafts, B, K, tokens);
  return hipGetLastError();
}
