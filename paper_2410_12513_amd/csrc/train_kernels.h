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
// (LM_COLS columns, all r rows) and the Bm rows of its row range in LDS once; a thread owns 8
// columns and walks the rows four at a time (four 16-byte loads of W in flight, every A value read
// from LDS serves four rows).  W is read and written exactly once.
constexpr int LM_COLS = 1024;      // columns per workgroup: 128 threads x 8 columns, two row groups at a time
constexpr int LM_RMAX = 32;        // largest rank (LDS: r * LM_COLS floats + the Bm rows)
constexpr int LM_RG = 4;           // rows per thread and iteration

template <typename WT>
__global__ void __launch_bounds__(WG) k_lora_merge(WT* __restrict__ W, const float* __restrict__ A, const float* __restrict__ Bm,
                                                   int n, int k, int r, float scale, int rows_per_wg) {
  extern __shared__ float lm_lds[];                      // A tile [r][LM_COLS], then Bm rows [rows_per_wg][r] (zero beyond n)
  float* a_lds = lm_lds;
  float* b_lds = lm_lds + r * LM_COLS;
  const int c0 = blockIdx.x * LM_COLS;
  const int row0 = blockIdx.y * rows_per_wg, row1 = min(n, row0 + rows_per_wg);
  for (int i = threadIdx.x; i < r * LM_COLS; i += WG) {
    const int j = i / LM_COLS, c = c0 + i % LM_COLS;
    a_lds[i] = c < k ? A[(size_t)j * k + c] : 0.f;
  }
  for (int i = threadIdx.x; i < rows_per_wg * r; i += WG)
    b_lds[i] = (row0 + i / r) < row1 ? Bm[(size_t)row0 * r + i] : 0.f;
  __syncthreads();
  const int tc = (threadIdx.x & 127) * 8, half = threadIdx.x >> 7;
  const int col = c0 + tc;
  if (col >= k) return;                                  // k is a multiple of 8: a thread's 8 columns are in or out together
  constexpr int NV = sizeof(WT) == 2 ? 1 : 2;            // 16-byte vectors per 8 elements
  for (int rb = half * LM_RG; row0 + rb < row1; rb += 2 * LM_RG) {
    uint4 raw[LM_RG][NV];
#pragma unroll
    for (int q = 0; q < LM_RG; ++q) {
      const int row = min(row0 + rb + q, row1 - 1);      // rows past the end re-read the last one and are not stored
      const uint4* w = reinterpret_cast<const uint4*>(W + (size_t)row * k + col);
#pragma unroll
      for (int v = 0; v < NV; ++v) raw[q][v] = w[v];
    }
    float acc[LM_RG][8];
#pragma unroll
    for (int q = 0; q < LM_RG; ++q)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[q][e] = 0.f;
    for (int j = 0; j < r; ++j) {
      const float4 a0 = *reinterpret_cast<const float4*>(a_lds + j * LM_COLS + tc);
      const float4 a1 = *reinterpret_cast<const float4*>(a_lds + j * LM_COLS + tc + 4);
      const float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
      for (int q = 0; q < LM_RG; ++q) {
        const float bj = b_lds[(rb + q) * r + j];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[q][e] = fmaf(bj, a[e], acc[q][e]);
      }
    }
#pragma unroll
    for (int q = 0; q < LM_RG; ++q) {
      const int row = row0 + rb + q;
      if (row >= row1) break;
      uint4* w = reinterpret_cast<uint4*>(W + (size_t)row * k + col);
      if constexpr (sizeof(WT) == 2) {
        const uint32_t u[4] = {raw[q][0].x, raw[q][0].y, raw[q][0].z, raw[q][0].w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t lo = f2bf(fmaf(scale, acc[q][2 * e], __uint_as_float(u[e] << 16)));
          const uint32_t hi = f2bf(fmaf(scale, acc[q][2 * e + 1], __uint_as_float(u[e] & 0xffff0000u)));
          o[e] = lo | (hi << 16);
        }
        w[0] = make_uint4(o[0], o[1], o[2], o[3]);
      } else {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          uint4 x = raw[q][v];
          x.x = __float_as_uint(fmaf(scale, acc[q][4 * v + 0], __uint_as_float(x.x)));
          x.y = __float_as_uint(fmaf(scale, acc[q][4 * v + 1], __uint_as_float(x.y)));
          x.z = __float_as_uint(fmaf(scale, acc[q][4 * v + 2], __uint_as_float(x.z)));
          x.w = __float_as_uint(fmaf(scale, acc[q][4 * v + 3], __uint_as_float(x.w)));
          w[v] = x;
        }
      }
    }
  }
}

}  // namespace first
