// Training-side forward pieces (Section 4.1: soft skip and the loss terms; Section 4.2: LoRA
// merged into the weights for inference).  Forward values only.
#pragma once
#include "common.h"

namespace first {

// Soft skip of one layer for one sequence: H = Hprev + rho * (H - Hprev), where Hprev is the
// stream that entered the layer, H holds Hprev + phi(Hprev) on entry, and rho is the router's
// score of Hprev (device scalar).
__global__ void __launch_bounds__(WG) k_soft_blend(float* __restrict__ H, const float* __restrict__ Hprev,
                                                   const float* __restrict__ rho, size_t n) {
  const float r = *rho;
  for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < n; i += (size_t)gridDim.x * WG) {
    const float p = Hprev[i];
    H[i] = fmaf(r, H[i] - p, p);
  }
}

// Cross entropy of one position per workgroup: ce[j] = log(sum_v exp(l[j][v])) - l[j][target[j]],
// 0 where target[j] < 0.  Three passes over the row (max, sum of exponentials, the pick), fp32.
__global__ void __launch_bounds__(WG) k_ce_rows(const float* __restrict__ logits, const int* __restrict__ targets,
                                                float* __restrict__ ce, int V) {
  __shared__ float red[WAVES];
  const int j = blockIdx.x;
  const int t = targets[j];
  if (t < 0 || t >= V) {
    if (threadIdx.x == 0) ce[j] = 0.f;
    return;
  }
  const float* row = logits + (size_t)j * V;
  float m = -INFINITY;
  for (int v = threadIdx.x; v < V; v += WG) m = fmaxf(m, row[v]);
  m = wave_max(m);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  m = red[0];
#pragma unroll
  for (int w = 1; w < WAVES; ++w) m = fmaxf(m, red[w]);
  float s = 0.f;
  for (int v = threadIdx.x; v < V; v += WG) s += expf(row[v] - m);
  const float tot = block_sum(s, red);
  if (threadIdx.x == 0) ce[j] = m + logf(tot) - row[t];
}

// The loss terms of one sequence (Section 4.1), one workgroup, fixed summation order:
//   terms[0] = L_CE  = mean of ce[j] over the positions with a target (0 when there is none)
//   terms[1] = L_Reg = sum over all router weights of w^2
//   terms[2] = L_PP  = sum_i rho[i]
//   terms[3] = L_CE + lambda * L_Reg + alpha * L_PP
__global__ void __launch_bounds__(WG) k_loss_terms(const float* __restrict__ ce, const int* __restrict__ targets, int T, int V,
                                                   const float* __restrict__ rho, int L, const float* __restrict__ router,
                                                   size_t n_router, float lambda, float alpha, float* __restrict__ terms) {
  __shared__ float red[WAVES];
  float s = 0.f, cnt = 0.f, q = 0.f;
  for (int j = threadIdx.x; j < T; j += WG) {
    const int t = targets[j];
    if (t >= 0 && t < V) { s += ce[j]; cnt += 1.f; }
  }
  for (size_t i = threadIdx.x; i < n_router; i += WG) q = fmaf(router[i], router[i], q);
  const float ce_sum = block_sum(s, red);
  const float n = block_sum(cnt, red);
  const float reg = block_sum(q, red);
  if (threadIdx.x == 0) {
    float pp = 0.f;
    for (int i = 0; i < L; ++i) pp += rho[i];
    const float l_ce = n > 0.f ? __fdiv_rn(ce_sum, n) : 0.f;
    terms[0] = l_ce; terms[1] = reg; terms[2] = pp;
    terms[3] = l_ce + lambda * reg + alpha * pp;
  }
}

// LoRA merge in place: W[row][col] += scale * sum_j Bm[row][j] * A[j][col]  (W [n, k] row-major in
// its storage type, Bm [n, r] and A [r, k] fp32).  The sum over j runs in fp32 in index order, the
// result is rounded once to the storage type.  A workgroup stages the A columns of its chunk
// (LM_COLS columns, all r rows) in LDS once and walks its share of the rows: W is read and
// written exactly once, A and Bm come from the caches.
constexpr int LM_COLS = 1024;      // columns per workgroup: 128 threads x 8 columns, two rows at a time
constexpr int LM_RMAX = 32;        // largest rank (LDS: r * LM_COLS floats)

template <typename WT>
__global__ void __launch_bounds__(WG) k_lora_merge(WT* __restrict__ W, const float* __restrict__ A, const float* __restrict__ Bm,
                                                   int n, int k, int r, float scale, int rows_per_wg) {
  extern __shared__ float a_lds[];                       // [r][LM_COLS]
  const int c0 = blockIdx.x * LM_COLS;
  for (int i = threadIdx.x; i < r * LM_COLS; i += WG) {
    const int j = i / LM_COLS, c = c0 + i % LM_COLS;
    a_lds[i] = c < k ? A[(size_t)j * k + c] : 0.f;
  }
  __syncthreads();
  const int tc = (threadIdx.x & 127) * 8, half = threadIdx.x >> 7;
  const int col = c0 + tc;
  const int row0 = blockIdx.y * rows_per_wg, row1 = min(n, row0 + rows_per_wg);
  if (col >= k) return;                                  // k is a multiple of 8: a thread's 8 columns are in or out together
  for (int row = row0 + half; row < row1; row += 2) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const float* b = Bm + (size_t)row * r;
    for (int j = 0; j < r; ++j) {
      const float bj = b[j];
      const float4 a0 = *reinterpret_cast<const float4*>(a_lds + j * LM_COLS + tc);
      const float4 a1 = *reinterpret_cast<const float4*>(a_lds + j * LM_COLS + tc + 4);
      acc[0] = fmaf(bj, a0.x, acc[0]); acc[1] = fmaf(bj, a0.y, acc[1]); acc[2] = fmaf(bj, a0.z, acc[2]); acc[3] = fmaf(bj, a0.w, acc[3]);
      acc[4] = fmaf(bj, a1.x, acc[4]); acc[5] = fmaf(bj, a1.y, acc[5]); acc[6] = fmaf(bj, a1.z, acc[6]); acc[7] = fmaf(bj, a1.w, acc[7]);
    }
    WT* w = W + (size_t)row * k + col;
    if constexpr (sizeof(WT) == 2) {
      float f[8];
      load_vec(w, f);
      uint16_t o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = f2bf(fmaf(scale, acc[e], f[e]));
      *reinterpret_cast<uint4*>(w) = make_uint4(o[0] | ((uint32_t)o[1] << 16), o[2] | ((uint32_t)o[3] << 16),
                                                o[4] | ((uint32_t)o[5] << 16), o[6] | ((uint32_t)o[7] << 16));
    } else {
      float4 w0 = *reinterpret_cast<const float4*>(w), w1 = *reinterpret_cast<const float4*>(w + 4);
      w0.x = fmaf(scale, acc[0], w0.x); w0.y = fmaf(scale, acc[1], w0.y); w0.z = fmaf(scale, acc[2], w0.z); w0.w = fmaf(scale, acc[3], w0.w);
      w1.x = fmaf(scale, acc[4], w1.x); w1.y = fmaf(scale, acc[5], w1.y); w1.z = fmaf(scale, acc[6], w1.z); w1.w = fmaf(scale, acc[7], w1.w);
      *reinterpret_cast<float4*>(w) = w0;
      *reinterpret_cast<float4*>(w + 4) = w1;
    }
  }
}

}  // namespace first
