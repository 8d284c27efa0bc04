// Temperature + top-k sampling over the logits of a decode step (Appendix, "Inference
// settings": temperature 0.8, top-k sampling over 10 tokens).  The draw itself is a uniform
// number in [0, 1) supplied by the caller, one per sequence: the library owns no random
// number generator.
//
//   candidates = the k largest logits, equal logits ordered by token index (lowest first);
//   p_j ~ exp((l_j - l_max) / T) over the candidates, summed in descending-logit order;
//   result = the first candidate whose cumulative weight exceeds u * total.
//
// Two stages: every workgroup of k_topk_part selects the top k of its 2048 logits (k rounds
// of "largest element after the previous one", values in registers); k_topk_sample merges the
// per-chunk lists of one sequence the same way and draws.  All fp32, fixed order.
#pragma once
#include "common.h"

namespace first {

constexpr int SMP_THREADS = 256;
constexpr int SMP_VPT = 8;                              // logits per thread in stage 1
constexpr int SMP_CHUNK = SMP_THREADS * SMP_VPT;
constexpr int SMP_KMAX = 64;
constexpr int SMP_NONE = 0x7fffffff;                    // index of "no candidate"

struct Cand { float v; int i; };

// a comes before b: larger logit, or equal logit and lower index
__device__ __forceinline__ bool cand_before(const Cand& a, const Cand& b) {
  return a.v > b.v || (a.v == b.v && a.i < b.i);
}

// The first candidate in order over the whole workgroup (every thread contributes one);
// red: SMP_THREADS / 64 entries of LDS.  Returns it in every thread.
__device__ __forceinline__ Cand wg_first(Cand c, Cand* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const Cand d{__shfl_xor(c.v, o, 64), __shfl_xor(c.i, o, 64)};
    if (cand_before(d, c)) c = d;
  }
  const int wave = threadIdx.x >> 6;
  __syncthreads();                                      // red may still be read from the round before
  if ((threadIdx.x & 63) == 0) red[wave] = c;
  __syncthreads();
  Cand r = red[0];
  for (int w = 1; w < SMP_THREADS / 64; ++w)
    if (cand_before(red[w], r)) r = red[w];
  return r;
}

// The draw: top[0..k) in order (SMP_NONE beyond the vocabulary), u in [0, 1).  One thread; every path that samples ends
// in this function, so that they take the same decision on the same candidates.
__device__ __forceinline__ int smp_draw(const Cand* top, int k, float temperature, float u) {
  int kk = 0;
  while (kk < k && top[kk].i != SMP_NONE) ++kk;
  const float lmax = top[0].v;
  float total = 0.f;
  for (int j = 0; j < kk; ++j) total += expf((top[j].v - lmax) / temperature);
  const float target = u * total;
  float cum = 0.f;
  int pick = kk > 0 ? top[kk - 1].i : 0;
  for (int j = 0; j < kk; ++j) {
    cum += expf((top[j].v - lmax) / temperature);
    if (cum > target) { pick = top[j].i; break; }
  }
  return pick;
}

// Stage 1.  grid (chunks, sequences).  part[(seq * chunks + chunk) * k + r] = r-th candidate of the chunk.
__global__ void __launch_bounds__(SMP_THREADS) k_topk_part(const float* __restrict__ logits, int V, int k, Cand* __restrict__ part) {
  __shared__ Cand red[SMP_THREADS / 64];
  const int tid = threadIdx.x, chunk = blockIdx.x, seq = blockIdx.y;
  const float* row = logits + (size_t)seq * V;
  Cand e[SMP_VPT];
#pragma unroll
  for (int j = 0; j < SMP_VPT; ++j) {
    const int idx = chunk * SMP_CHUNK + j * SMP_THREADS + tid;
    e[j] = idx < V ? Cand{row[idx], idx} : Cand{-INFINITY, SMP_NONE};
  }
  Cand last{INFINITY, -1};
  Cand* out = part + ((size_t)seq * gridDim.x + chunk) * k;
  for (int r = 0; r < k; ++r) {
    Cand best{-INFINITY, SMP_NONE};
#pragma unroll
    for (int j = 0; j < SMP_VPT; ++j)
      if (e[j].i != SMP_NONE && cand_before(last, e[j]) && cand_before(e[j], best)) best = e[j];
    best = wg_first(best, red);
    if (tid == 0) out[r] = best;
    last = best.i == SMP_NONE ? Cand{-INFINITY, SMP_NONE} : best;   // nothing left: nothing comes after
  }
}

// Stage 2.  grid (sequences).  n = chunks * k candidates of the sequence.
__global__ void __launch_bounds__(SMP_THREADS) k_topk_sample(const Cand* __restrict__ part, int n, int k, float temperature,
                                                            const float* __restrict__ uniforms, int* __restrict__ token_out,
                                                            int* __restrict__ cand_out) {
  __shared__ Cand red[SMP_THREADS / 64];
  __shared__ Cand top[SMP_KMAX];
  const int tid = threadIdx.x, seq = blockIdx.x;
  const Cand* c = part + (size_t)seq * n;
  Cand last{INFINITY, -1};
  for (int r = 0; r < k; ++r) {
    Cand best{-INFINITY, SMP_NONE};
    for (int j = tid; j < n; j += SMP_THREADS) {
      const Cand x = c[j];
      if (x.i != SMP_NONE && cand_before(last, x) && cand_before(x, best)) best = x;
    }
    best = wg_first(best, red);
    if (tid == 0) top[r] = best;
    last = best.i == SMP_NONE ? Cand{-INFINITY, SMP_NONE} : best;
  }
  __syncthreads();
  if (tid < k && cand_out != nullptr) cand_out[(size_t)seq * k + tid] = top[tid].i == SMP_NONE ? -1 : top[tid].i;
  if (tid == 0) token_out[seq] = smp_draw(top, k, temperature, uniforms[seq]);
}

}  // namespace first
