// Prefill kernels: every layer runs on the whole prompt (Section 4.3 item 1), the routers
// are scored on the stream entering each layer (Section 4.1), KV of all layers is written.
#pragma once
#include "common.h"

namespace first {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;

// H[t] = E[ids[t]] widened to fp32.  grid = T.
template <typename WT>
__global__ void __launch_bounds__(WG) k_embed_rows(const int* __restrict__ ids, const WT* __restrict__ E,
                                                   float* __restrict__ H, int D, int V) {
  const int t = blockIdx.x;
  int tok = ids[t];
  tok = min(max(tok, 0), V - 1);
  const WT* row = E + (size_t)tok * D;
  for (int k = threadIdx.x; k < D; k += WG) H[(size_t)t * D + k] = to_f32(row[k]);
}

// cs[t][i] = (cos, sin)(t * theta_i), angle formed in fp64.  grid covers T*half threads.
__global__ void __launch_bounds__(WG) k_rope_table(const double* __restrict__ theta, float2* __restrict__ cs,
                                                   int T, int half) {
  const int i = blockIdx.x * WG + threadIdx.x;
  if (i >= T * half) return;
  const int t = i / half, d = i - t * half;
  const double a = (double)t * theta[d];
  cs[i] = make_float2((float)cos(a), (float)sin(a));
}

// One wave per token: x = RMSNorm(H[t]; gain) in the GEMM input type, and, if rw is given,
// sig[t] = sigmoid(rw . H[t]) on the raw stream (router, Section 4.1).  grid = ceil(T/4).
template <typename XT>
__global__ void __launch_bounds__(WG) k_rmsnorm_router(const float* __restrict__ H, const float* __restrict__ gain,
                                                       const float* __restrict__ rw, XT* __restrict__ x,
                                                       float* __restrict__ sig, int T, int D, float eps,
                                                       bf16* __restrict__ xh = nullptr, bf16* __restrict__ xl = nullptr) {
  const int t = blockIdx.x * WAVES + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (t >= T) return;
  const float* row = H + (size_t)t * D;
  // Eight 16-byte pieces of the row per lane and round, all requested before the first is used (one piece per round
  // is one memory round trip per round); same order of additions as a piece-by-piece loop.
  constexpr int RB = 8;
  float ss = 0.f, dot = 0.f;
  for (int k0 = lane * 4; k0 < D; k0 += 256 * RB) {
    float4 v[RB], w[RB];
#pragma unroll
    for (int u = 0; u < RB; ++u) {
      const int k = min(k0 + 256 * u, D - 4);
      v[u] = *reinterpret_cast<const float4*>(row + k);
      w[u] = rw ? *reinterpret_cast<const float4*>(rw + k) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < RB; ++u) {
      if (k0 + 256 * u < D) {
        ss = fmaf(v[u].x, v[u].x, ss); ss = fmaf(v[u].y, v[u].y, ss); ss = fmaf(v[u].z, v[u].z, ss); ss = fmaf(v[u].w, v[u].w, ss);
        dot = fmaf(v[u].x, w[u].x, dot); dot = fmaf(v[u].y, w[u].y, dot); dot = fmaf(v[u].z, w[u].z, dot); dot = fmaf(v[u].w, w[u].w, dot);
      }
    }
  }
  ss = wave_sum(ss);
  const float r = 1.0f / sqrtf(ss / (float)D + eps);
#pragma unroll 4
  for (int k = lane * 4; k < D; k += 256) {
    const float4 v = *reinterpret_cast<const float4*>(row + k);
    const float4 g = *reinterpret_cast<const float4*>(gain + k);
    const float y[4] = {v.x * g.x * r, v.y * g.y * r, v.z * g.z * r, v.w * g.w * r};
    if (xh) {                                      // split for the matrix cores: y = hi + lo
      uint16_t hi[4], lo[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) { hi[e] = f2bf(y[e]); lo[e] = f2bf(y[e] - bf2f(hi[e])); }
      *reinterpret_cast<uint2*>(xh + (size_t)t * D + k) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
      *reinterpret_cast<uint2*>(xl + (size_t)t * D + k) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
    } else {
      XT* o = x + (size_t)t * D + k;
      o[0] = from_f32<XT>(y[0]); o[1] = from_f32<XT>(y[1]); o[2] = from_f32<XT>(y[2]); o[3] = from_f32<XT>(y[3]);
    }
  }
  if (rw) {
    dot = wave_sum(dot);
    if (lane == 0) sig[t] = sigmoidf(dot);
  }
}

// rho = mean_t sig[t] (fixed summation order); mask = (rho >= 0.5).  One workgroup.
__global__ void __launch_bounds__(WG) k_router_reduce(const float* __restrict__ sig, int T,
                                                      float* __restrict__ rho, uint8_t* __restrict__ mask) {
  __shared__ float red[WAVES];
  float s = 0.f;
  for (int t = threadIdx.x; t < T; t += WG) s += sig[t];
  const float tot = block_sum(s, red);
  if (threadIdx.x == 0) {
    const float r = __fdiv_rn(tot, (float)T);
    *rho = r;
    *mask = (r >= 0.5f) ? 1 : 0;
  }
}

// kept = ascending indices of set mask bytes; one wave per sequence (ballot + popcount).
__global__ void __launch_bounds__(64) k_compact(const uint8_t* __restrict__ mask, int L, int* __restrict__ kept,
                                                int* __restrict__ n_kept) {
  const int b = blockIdx.x, lane = threadIdx.x;
  int base = 0;
  for (int i0 = 0; i0 < L; i0 += 64) {
    const int i = i0 + lane;
    const bool on = (i < L) && mask[(size_t)b * L + i] != 0;
    const unsigned long long bal = __ballot(on);
    if (on) kept[(size_t)b * L + base + __popcll(bal & ((1ull << lane) - 1ull))] = i;
    base += __popcll(bal);
  }
  for (int i = base + lane; i < L; i += 64) kept[(size_t)b * L + i] = -1;
  if (lane == 0) n_kept[b] = base;
}

// ---------------------------------------------------------------------------------------
// C[M,N] (+)= A[M,K] . W[N,K]^T, bf16 inputs, fp32 accumulate on the matrix cores.
// 128x128 tile per workgroup, 4 waves of 64x64 (2x2 MFMA 32x32x16), K step 64, operands
// staged through LDS with the next tile prefetched into registers.
constexpr int GB_M = 128, GB_N = 128, GB_K = 64, GB_PITCH = GB_K + 8;

__global__ void __launch_bounds__(WG) k_gemm_nt_bf16(const bf16* __restrict__ A, const bf16* __restrict__ W,
                                                     float* __restrict__ C, int M, int N, int K, int accumulate) {
  __shared__ __align__(16) uint16_t sA[GB_M * GB_PITCH];
  __shared__ __align__(16) uint16_t sB[GB_N * GB_PITCH];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int m0 = blockIdx.y * GB_M, n0 = blockIdx.x * GB_N;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  floatx16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[4], rb[4];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = tid + WG * i, row = v >> 3, kc = (v & 7) << 3;
      const int k = k0 + kc;
      ra[i] = make_uint4(0, 0, 0, 0);
      rb[i] = make_uint4(0, 0, 0, 0);
      if (k < K) {
        if (m0 + row < M) ra[i] = *reinterpret_cast<const uint4*>(A + (size_t)(m0 + row) * K + k);
        if (n0 + row < N) rb[i] = *reinterpret_cast<const uint4*>(W + (size_t)(n0 + row) * K + k);
      }
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = tid + WG * i, row = v >> 3, kc = (v & 7) << 3;
      *reinterpret_cast<uint4*>(sA + row * GB_PITCH + kc) = ra[i];
      *reinterpret_cast<uint4*>(sB + row * GB_PITCH + kc) = rb[i];
    }
  };

  fetch(0);
  for (int k0 = 0; k0 < K; k0 += GB_K) {
    __syncthreads();
    stash();
    __syncthreads();
    if (k0 + GB_K < K) fetch(k0 + GB_K);
#pragma unroll
    for (int kk = 0; kk < GB_K; kk += 16) {
      bf16x8_t a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = *reinterpret_cast<const bf16x8_t*>(sA + (wm + i * 32 + (lane & 31)) * GB_PITCH + kk + ((lane >> 5) << 3));
        b[i] = *reinterpret_cast<const bf16x8_t*>(sB + (wn + i * 32 + (lane & 31)) * GB_PITCH + kk + ((lane >> 5) << 3));
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }
  // D layout of the 32x32 MFMA: lane -> column (lane & 31); register r -> row
  // 8*(r/4) + 4*(lane/32) + r%4.
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < M && col < N) {
          float* c = C + (size_t)row * N + col;
          *c = accumulate ? *c + acc[i][j][r] : acc[i][j][r];
        }
      }
    }
}

// Same contraction with fp32 activations A and bf16 weights W.  Each activation is split into
// two bf16 numbers, a = hi + lo with hi = bf16(a) and lo = bf16(a - hi), and both parts go
// through the matrix cores against the same weight tile, so the product carries about 16
// mantissa bits of the activation instead of 8 (the weights are bf16 exactly).  This keeps
// the prompt's hidden states, KV and first-token logits close to full-precision arithmetic
// at twice the matrix-core work.
__global__ void __launch_bounds__(WG) k_gemm_nt_bf16_split(const float* __restrict__ A, const bf16* __restrict__ W,
                                                           float* __restrict__ C, int M, int N, int K, int accumulate) {
  __shared__ __align__(16) uint16_t sAh[GB_M * GB_PITCH];
  __shared__ __align__(16) uint16_t sAl[GB_M * GB_PITCH];
  __shared__ __align__(16) uint16_t sB[GB_N * GB_PITCH];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int m0 = blockIdx.y * GB_M, n0 = blockIdx.x * GB_N;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  floatx16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float4 ra[4][2];
  uint4 rb[4];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = tid + WG * i, row = v >> 3, kc = (v & 7) << 3;
      const int k = k0 + kc;
      ra[i][0] = make_float4(0, 0, 0, 0); ra[i][1] = make_float4(0, 0, 0, 0);
      rb[i] = make_uint4(0, 0, 0, 0);
      if (k < K) {
        if (m0 + row < M) {
          ra[i][0] = *reinterpret_cast<const float4*>(A + (size_t)(m0 + row) * K + k);
          ra[i][1] = *reinterpret_cast<const float4*>(A + (size_t)(m0 + row) * K + k + 4);
        }
        if (n0 + row < N) rb[i] = *reinterpret_cast<const uint4*>(W + (size_t)(n0 + row) * K + k);
      }
    }
  };
  auto split2 = [](float a, float b, uint32_t& hi, uint32_t& lo) {
    const uint32_t ha = f2bf(a), hb = f2bf(b);
    hi = ha | (hb << 16);
    lo = (uint32_t)f2bf(a - bf2f(ha)) | ((uint32_t)f2bf(b - bf2f(hb)) << 16);
  };
  auto stash = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int v = tid + WG * i, row = v >> 3, kc = (v & 7) << 3;
      uint4 h, l;
      split2(ra[i][0].x, ra[i][0].y, h.x, l.x); split2(ra[i][0].z, ra[i][0].w, h.y, l.y);
      split2(ra[i][1].x, ra[i][1].y, h.z, l.z); split2(ra[i][1].z, ra[i][1].w, h.w, l.w);
      *reinterpret_cast<uint4*>(sAh + row * GB_PITCH + kc) = h;
      *reinterpret_cast<uint4*>(sAl + row * GB_PITCH + kc) = l;
      *reinterpret_cast<uint4*>(sB + row * GB_PITCH + kc) = rb[i];
    }
  };

  fetch(0);
  for (int k0 = 0; k0 < K; k0 += GB_K) {
    __syncthreads();
    stash();
    __syncthreads();
    if (k0 + GB_K < K) fetch(k0 + GB_K);
#pragma unroll
    for (int kk = 0; kk < GB_K; kk += 16) {
      bf16x8_t ah[2], al[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int ao = (wm + i * 32 + (lane & 31)) * GB_PITCH + kk + ((lane >> 5) << 3);
        ah[i] = *reinterpret_cast<const bf16x8_t*>(sAh + ao);
        al[i] = *reinterpret_cast<const bf16x8_t*>(sAl + ao);
        b[i] = *reinterpret_cast<const bf16x8_t*>(sB + (wn + i * 32 + (lane & 31)) * GB_PITCH + kk + ((lane >> 5) << 3));
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], b[j], acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], b[j], acc[i][j], 0, 0, 0);
        }
    }
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < M && col < N) {
          float* c = C + (size_t)row * N + col;
          *c = accumulate ? *c + acc[i][j][r] : acc[i][j][r];
        }
      }
    }
}

// The same split-precision contraction with the activations already split by their producer
// (Ah + Al, bf16 each): no conversion work here, which otherwise repeats once per column tile.
// A 16-byte global load whose destination the compiler must treat as in use from here on (it is written when the load
// lands), a wait that leaves the N youngest loads of the wave outstanding, and the point from which a destination
// may be read.  A kernel using these must not spill registers (see build.py).
__device__ __forceinline__ void pf_issue16(u32x4_t& v, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p) : "memory");
}
template <int N> __device__ __forceinline__ void pf_wait() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void pf_use(u32x4_t& v) { asm volatile("" : "+v"(v)); }

// BM x BN output tile per workgroup, the four waves arranged WGM x WGN over it (wave tile = (BM / WGM) x (BN / WGN),
// a multiple of 32 x 32 each way).
// GU: the B tile is BN / 2 rows of W (gate) followed by the same BN / 2 rows of W2 (up); instead of storing C the
// epilogue forms SiLU(gate) * up for the tile's BM x BN / 2 outputs and writes them split into zh + zl ([M, N] bf16 each).
template <int BM, int BN, int WGM, int WGN, int NSTG = 2, bool GU = false>
__device__ __forceinline__ void gemm_nt_bf16_hl_tile(const bf16* __restrict__ Ah, const bf16* __restrict__ Al,
                                                     const bf16* __restrict__ W, float* __restrict__ C, int M, int N,
                                                     int K, int accumulate, int m0, int n0,
                                                     const bf16* __restrict__ W2 = nullptr, bf16* __restrict__ zh = nullptr,
                                                     bf16* __restrict__ zl = nullptr) {
  static_assert(WGM * WGN == WAVES, "four waves");
  constexpr int TM = BM / WGM, TN = BN / WGN, IM = TM / 32, JN = TN / 32;
  constexpr int VA = BM * 8 / WG, VB = BN * 8 / WG;            // 16-byte vectors per thread and K step
  static_assert(TM % 32 == 0 && TN % 32 == 0 && VA >= 1 && VB >= 1, "tile shape");
  __shared__ __align__(16) uint16_t sAll[(2 * BM + BN) * GB_PITCH];     // one block: the GU epilogue reuses it
  uint16_t* sAh = sAll;
  uint16_t* sAl = sAll + BM * GB_PITCH;
  uint16_t* sB = sAll + 2 * BM * GB_PITCH;
  static_assert(!GU || (WGN == 2 && VB % 2 == 0 && (size_t)BM * (BN / 2) * 4 <= sizeof(sAll)), "gate columns | up columns");
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = (wave / WGN) * TM, wn = (wave % WGN) * TN;
  floatx16_t acc[IM][JN];
#pragma unroll
  for (int i = 0; i < IM; ++i)
#pragma unroll
    for (int j = 0; j < JN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Two K steps of operands are in flight in registers: a load takes longer than the matrix cores need for one step.
  // The loads are issued through inline asm and waited for by count (the compiler would sink ordinary loads down to
  // their first use and wait for all of them at every barrier): rows and K offsets past the end are clamped for the
  // load and zeroed when the registers go to LDS, the step count is rounded up to a multiple of the stages, the barriers wait for LDS
  // only, and pf_wait<NL> lets exactly the other stage's NL loads stay outstanding (loads return in order).
  struct Stage { u32x4_t h[VA], l[VA], b[VB]; };
  constexpr int NL = 2 * VA + VB;
  const int nsteps = (K + GB_K - 1) / GB_K;
  auto fetch = [&](Stage& R, int step) __attribute__((always_inline)) {
    const int k0 = min(step, nsteps - 1) * GB_K;
#pragma unroll
    for (int i = 0; i < VA; ++i) {
      const int v = tid + WG * i, row = min(m0 + (v >> 3), M - 1), k = min(k0 + ((v & 7) << 3), K - 8);
      pf_issue16(R.h[i], Ah + (size_t)row * K + k);
      pf_issue16(R.l[i], Al + (size_t)row * K + k);
    }
#pragma unroll
    for (int i = 0; i < VB; ++i) {
      const int v = tid + WG * i, k = min(k0 + ((v & 7) << 3), K - 8);
      if (GU) {                                        // rows 0 .. BN/2-1 of the tile: gate, the rest: up (i decides)
        const int row = min(n0 + ((v >> 3) & (BN / 2 - 1)), N - 1);
        pf_issue16(R.b[i], (i < VB / 2 ? W : W2) + (size_t)row * K + k);
      } else {
        const int row = min(n0 + (v >> 3), N - 1);
        pf_issue16(R.b[i], W + (size_t)row * K + k);
      }
    }
  };
  auto stash = [&](Stage& R, int step) __attribute__((always_inline)) {
    const int k0 = step * GB_K;
    const u32x4_t zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < VA; ++i) {
      const int v = tid + WG * i, row = v >> 3, kc = (v & 7) << 3;
      const bool ok = step < nsteps && k0 + kc < K && m0 + row < M;
      pf_use(R.h[i]); pf_use(R.l[i]);
      *reinterpret_cast<u32x4_t*>(sAh + row * GB_PITCH + kc) = ok ? R.h[i] : zero;
      *reinterpret_cast<u32x4_t*>(sAl + row * GB_PITCH + kc) = ok ? R.l[i] : zero;
    }
#pragma unroll
    for (int i = 0; i < VB; ++i) {
      const int v = tid + WG * i, row = v >> 3, kc = (v & 7) << 3;
      const bool ok = step < nsteps && k0 + kc < K && n0 + (GU ? (row & (BN / 2 - 1)) : row) < N;
      pf_use(R.b[i]);
      *reinterpret_cast<u32x4_t*>(sB + row * GB_PITCH + kc) = ok ? R.b[i] : zero;
    }
  };
  auto compute = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < GB_K; kk += 16) {
      bf16x8_t ah[IM], al[IM], b[JN];
#pragma unroll
      for (int i = 0; i < IM; ++i) {
        const int ao = (wm + i * 32 + (lane & 31)) * GB_PITCH + kk + ((lane >> 5) << 3);
        ah[i] = *reinterpret_cast<const bf16x8_t*>(sAh + ao);
        al[i] = *reinterpret_cast<const bf16x8_t*>(sAl + ao);
      }
#pragma unroll
      for (int j = 0; j < JN; ++j)
        b[j] = *reinterpret_cast<const bf16x8_t*>(sB + (wn + j * 32 + (lane & 31)) * GB_PITCH + kk + ((lane >> 5) << 3));
      // low halves first, then high halves: two products into the same accumulator are never issued back to back
#pragma unroll
      for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < JN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], b[j], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < JN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  // NSTG stages (K steps) of operands in flight; the loop is unrolled over the stages so that every stage is a fixed
  // set of registers.
  Stage R[NSTG];
#pragma unroll
  for (int q = 0; q < NSTG; ++q) fetch(R[q], q);
  for (int s = 0; s < nsteps; s += NSTG) {
#pragma unroll
    for (int q = 0; q < NSTG; ++q) {
      lds_barrier();                       // everyone has read the previous step's tiles
      pf_wait<NL * (NSTG - 1)>();          // this stage has landed; the younger ones may still be on their way
      stash(R[q], s + q);
      lds_barrier();
      fetch(R[q], s + q + NSTG);
      compute();
    }
  }
  // The last fetches (clamped re-loads nobody reads) are still on their way: wait for them, and only then let go of
  // their destinations - the compiler would otherwise hand those registers to the epilogue's addresses while the loads
  // can still land in them.
  pf_wait<0>();
#pragma unroll
  for (int q = 0; q < NSTG; ++q) {
#pragma unroll
    for (int i = 0; i < VA; ++i) { pf_use(R[q].h[i]); pf_use(R[q].l[i]); }
#pragma unroll
    for (int i = 0; i < VB; ++i) pf_use(R[q].b[i]);
  }
  if constexpr (GU) {
    // the up waves (wn != 0) pass their accumulators through LDS to the gate waves of the same rows
    float* u_lds = reinterpret_cast<float*>(sAll);                 // [BM][BN / 2]
    lds_barrier();                                                 // every wave has finished reading the operand tiles
    if (wn != 0) {
#pragma unroll
      for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < JN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            u_lds[(wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * (BN / 2) + j * 32 + (lane & 31)] = acc[i][j][r];
    }
    lds_barrier();
    if (wn == 0) {
#pragma unroll
      for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < JN; ++j) {
          const int col = n0 + j * 32 + (lane & 31);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int rl = wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3), row = m0 + rl;
            if (row < M && col < N) {
              const float z = siluf(acc[i][j][r]) * u_lds[rl * (BN / 2) + j * 32 + (lane & 31)];
              const bf16 h = from_f32<bf16>(z);
              zh[(size_t)row * N + col] = h;
              zl[(size_t)row * N + col] = from_f32<bf16>(z - to_f32(h));
            }
          }
        }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < IM; ++i)
#pragma unroll
    for (int j = 0; j < JN; ++j) {
      const int col = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < M && col < N) {
          float* c = C + (size_t)row * N + col;
          *c = accumulate ? *c + acc[i][j][r] : acc[i][j][r];
        }
      }
    }
}

__global__ void __launch_bounds__(WG) k_gemm_nt_bf16_hl(const bf16* __restrict__ Ah, const bf16* __restrict__ Al,
                                                        const bf16* __restrict__ W, float* __restrict__ C, int M, int N,
                                                        int K, int accumulate) {
  gemm_nt_bf16_hl_tile<GB_M, GB_N, 2, 2>(Ah, Al, W, C, M, N, K, accumulate, blockIdx.y * GB_M, blockIdx.x * GB_N);
}

// The same with 64-row tiles, for shapes whose 128 x 128 tiles would leave every compute unit a single workgroup
// (one wave per SIMD, nothing to overlap a barrier or a load with): twice the workgroups, two per compute unit.
constexpr int GB_MS = 64;
__global__ void __launch_bounds__(WG) k_gemm_nt_bf16_hl_s(const bf16* __restrict__ Ah, const bf16* __restrict__ Al,
                                                          const bf16* __restrict__ W, float* __restrict__ C, int M, int N,
                                                          int K, int accumulate) {
  gemm_nt_bf16_hl_tile<GB_MS, GB_N, 2, 2>(Ah, Al, W, C, M, N, K, accumulate, blockIdx.y * GB_MS, blockIdx.x * GB_N);
}

// Several weight matrices applied to the same activations in one launch (Q, K and V; gate and up): the column
// blocks of the segments follow each other in blockIdx.x, each segment with its own matrix, output and width.
// A matrix of 1024 rows alone is 64 workgroups at 1024 tokens - a quarter of the compute units; together the
// projections of one input fill whole rounds.
struct GemmSeg { const bf16* W; float* C; int N; int blocks; };     // blocks = ceil(N / GB_N)
struct GemmSegs { GemmSeg s[3]; int n; };
__global__ void __launch_bounds__(WG) k_gemm_nt_bf16_hl_seg(const bf16* __restrict__ Ah, const bf16* __restrict__ Al,
                                                            GemmSegs segs, int M, int K, int accumulate) {
  int bx = blockIdx.x, i = 0;
  while (i + 1 < segs.n && bx >= segs.s[i].blocks) { bx -= segs.s[i].blocks; ++i; }
  const GemmSeg g = segs.s[i];
  gemm_nt_bf16_hl_tile<GB_M, GB_N, 2, 2>(Ah, Al, g.W, g.C, M, g.N, K, accumulate, blockIdx.y * GB_M, bx * GB_N);
}

// Gate and up projections with SiLU(gate) * up in the epilogue: a workgroup takes 64 columns of both matrices for its
// 128 rows, so the MLP activation leaves the GEMM already split for the down projection - no fp32 gate / up
// matrices in memory and no elementwise launch.  N = d_ffn.
__global__ void __launch_bounds__(WG) k_gemm_nt_bf16_hl_gu(const bf16* __restrict__ Ah, const bf16* __restrict__ Al,
                                                           const bf16* __restrict__ Wg, const bf16* __restrict__ Wu,
                                                           bf16* __restrict__ zh, bf16* __restrict__ zl, int M, int N, int K) {
  gemm_nt_bf16_hl_tile<GB_M, GB_N, 2, 2, 2, true>(Ah, Al, Wg, nullptr, M, N, K, 0, blockIdx.y * GB_M, blockIdx.x * (GB_N / 2), Wu,
                                                  zh, zl);
}

// fp32 variant (the small full-precision configuration): 64x64 tile, 4x4 per thread.
__global__ void __launch_bounds__(WG) k_gemm_nt_f32(const float* __restrict__ A, const float* __restrict__ W,
                                                    float* __restrict__ C, int M, int N, int K, int accumulate) {
  __shared__ __align__(16) float sA[16][68];
  __shared__ __align__(16) float sB[16][68];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int lr = tid >> 2, lk = (tid & 3) << 2;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    float4 va = make_float4(0, 0, 0, 0), vb = make_float4(0, 0, 0, 0);
    if (k0 + lk < K) {
      if (m0 + lr < M) va = *reinterpret_cast<const float4*>(A + (size_t)(m0 + lr) * K + k0 + lk);
      if (n0 + lr < N) vb = *reinterpret_cast<const float4*>(W + (size_t)(n0 + lr) * K + k0 + lk);
    }
    __syncthreads();
    sA[lk][lr] = va.x; sA[lk + 1][lr] = va.y; sA[lk + 2][lr] = va.z; sA[lk + 3][lr] = va.w;
    sB[lk][lr] = vb.x; sB[lk + 1][lr] = vb.y; sB[lk + 2][lr] = vb.z; sB[lk + 3][lr] = vb.w;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&sA[k][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&sB[k][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
      if (row < M && col < N) {
        float* c = C + (size_t)row * N + col;
        *c = accumulate ? *c + acc[i][j] : acc[i][j];
      }
    }
}

// ---------------------------------------------------------------------------------------
// Per token: rotate q (in place, pre-scaled by 1/sqrt(hd)), rotate k, round k and v to the
// cache type and write them to the token's page slot.  grid = T.
template <typename KVT>
__global__ void __launch_bounds__(WG) k_rope_kvwrite(float* __restrict__ q, const float* __restrict__ kraw,
                                                     const float* __restrict__ vraw, const float2* __restrict__ cs,
                                                     const int* __restrict__ pt, KVT* __restrict__ pool,
                                                     size_t page_elems, int Hq, int Hkv, int hd, int P, float qscale) {
  const int t = blockIdx.x, half = hd >> 1;
  const float2* c = cs + (size_t)t * half;
  float* qrow = q + (size_t)t * Hq * hd;
  for (int i = threadIdx.x; i < Hq * half; i += WG) {
    const int h = i / half, d = i - h * half;
    const float x1 = qrow[h * hd + d], x2 = qrow[h * hd + d + half];
    qrow[h * hd + d] = (x1 * c[d].x - x2 * c[d].y) * qscale;
    qrow[h * hd + d + half] = (x2 * c[d].x + x1 * c[d].y) * qscale;
  }
  const size_t base = (size_t)pt[t / P] * page_elems + (size_t)(t % P) * hd;
  const size_t v_off = (size_t)Hkv * P * hd;
  const float* krow = kraw + (size_t)t * Hkv * hd;
  const float* vrow = vraw + (size_t)t * Hkv * hd;
  for (int i = threadIdx.x; i < Hkv * half; i += WG) {
    const int g = i / half, d = i - g * half;
    const float x1 = krow[g * hd + d], x2 = krow[g * hd + d + half];
    KVT* dst = pool + base + (size_t)g * P * hd;
    dst[d] = from_f32<KVT>(x1 * c[d].x - x2 * c[d].y);
    dst[d + half] = from_f32<KVT>(x2 * c[d].x + x1 * c[d].y);
  }
  for (int i = threadIdx.x; i < Hkv * hd; i += WG) {
    const int g = i / hd, d = i - g * hd;
    pool[base + v_off + (size_t)g * P * hd + d] = from_f32<KVT>(vrow[i]);
  }
}

// Causal GQA attention over the prompt, reading K and V back from the cache pages.
// grid = (ceil(T/QB), Hkv); the workgroup owns QB query positions x G heads (<= 64 rows),
// one wave per row in turn; 64-key tiles of K (padded rows) and V are shared through LDS.
constexpr int PA_RPW = 16;      // rows per wave
template <typename XT, typename KVT>
__global__ void __launch_bounds__(WG) k_attn_prefill(const float* __restrict__ q, XT* __restrict__ out,
                                                     const int* __restrict__ pt, const KVT* __restrict__ pool,
                                                     size_t page_elems, int T, int Hq, int Hkv, int hd, int P, int QB) {
  extern __shared__ __align__(16) float smem_f[];
  constexpr int VEC = Vec<KVT>::N;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int G = Hq / Hkv, g = blockIdx.y, t0 = blockIdx.x * QB;
  const int NR = QB * G;
  float* qs = smem_f;                                              // [NR][hd]
  char* kt = reinterpret_cast<char*>(qs + 64 * hd);
  const int kpitch = hd * (int)sizeof(KVT) + 4;
  const KVT* vt = reinterpret_cast<const KVT*>(kt + 64 * kpitch);
  KVT* vtw = reinterpret_cast<KVT*>(kt + 64 * kpitch);
  const size_t head_off = (size_t)g * P * hd, v_off = (size_t)Hkv * P * hd;

  for (int i = tid; i < NR * hd; i += WG) {
    const int rr = i / hd, d = i - rr * hd;
    const int t = t0 + rr / G, H = g * G + rr % G;
    qs[i] = (t < T) ? q[((size_t)t * Hq + H) * hd + d] : 0.f;
  }
  float m[PA_RPW], l[PA_RPW], o0[PA_RPW], o1[PA_RPW];
#pragma unroll
  for (int i = 0; i < PA_RPW; ++i) { m[i] = -INFINITY; l[i] = 0.f; o0[i] = 0.f; o1[i] = 0.f; }

  const int k_end = min(T, t0 + QB);
  const int vec_per_key = hd / VEC;
  for (int kt0 = 0; kt0 < k_end; kt0 += 64) {
    __syncthreads();
    for (int i = tid; i < 64 * vec_per_key; i += WG) {
      const int j = i / vec_per_key, c = (i - j * vec_per_key) * VEC;
      const int key = kt0 + j;
      uint4 kv4 = make_uint4(0, 0, 0, 0), vv4 = make_uint4(0, 0, 0, 0);
      if (key < k_end) {
        const size_t base = (size_t)pt[key / P] * page_elems + head_off + (size_t)(key % P) * hd + c;
        kv4 = *reinterpret_cast<const uint4*>(pool + base);
        vv4 = *reinterpret_cast<const uint4*>(pool + base + v_off);
      }
      uint32_t* kd = reinterpret_cast<uint32_t*>(kt + j * kpitch + c * sizeof(KVT));
      kd[0] = kv4.x; kd[1] = kv4.y; kd[2] = kv4.z; kd[3] = kv4.w;
      *reinterpret_cast<uint4*>(vtw + j * hd + c) = vv4;
    }
    __syncthreads();
#pragma unroll
    for (int ri = 0; ri < PA_RPW; ++ri) {
      const int rr = wave + ri * WAVES;
      const int t = t0 + rr / G;
      if (rr < NR && t < T && kt0 <= t) {
        const int jn = min(64, t - kt0 + 1);
        float sc = 0.f;
        const char* krow = kt + lane * kpitch;
        const float* qv = qs + rr * hd;
        if (sizeof(KVT) == 2) {
          for (int d = 0; d < hd; d += 2) {
            const uint32_t w2 = *reinterpret_cast<const uint32_t*>(krow + d * 2);
            sc = fmaf(qv[d], __uint_as_float(w2 << 16), sc);
            sc = fmaf(qv[d + 1], __uint_as_float(w2 & 0xffff0000u), sc);
          }
        } else {
          for (int d = 0; d < hd; ++d) sc = fmaf(qv[d], *reinterpret_cast<const float*>(krow + d * 4), sc);
        }
        if (lane >= jn) sc = -INFINITY;
        const float mn = fmaxf(m[ri], wave_max(sc));
        const float corr = expf(m[ri] - mn);
        const float pj = (lane < jn) ? expf(sc - mn) : 0.f;
        l[ri] = l[ri] * corr + wave_sum(pj);
        o0[ri] *= corr; o1[ri] *= corr;
        m[ri] = mn;
        for (int j = 0; j < jn; ++j) {
          const float pb = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pj), j));
          if (lane < hd) o0[ri] = fmaf(pb, to_f32(vt[j * hd + lane]), o0[ri]);
          if (lane + 64 < hd) o1[ri] = fmaf(pb, to_f32(vt[j * hd + lane + 64]), o1[ri]);
        }
      }
    }
  }
#pragma unroll
  for (int ri = 0; ri < PA_RPW; ++ri) {
    const int rr = wave + ri * WAVES;
    const int t = t0 + rr / G, H = g * G + rr % G;
    if (rr < NR && t < T) {
      XT* o = out + ((size_t)t * Hq + H) * hd;
      if (lane < hd) o[lane] = from_f32<XT>(o0[ri] / l[ri]);
      if (lane + 64 < hd) o[lane + 64] = from_f32<XT>(o1[ri] / l[ri]);
    }
  }
}

// z = silu(g) * u in the GEMM input type.
template <typename XT>
__global__ void __launch_bounds__(WG) k_silu_mul(const float* __restrict__ g, const float* __restrict__ u,
                                                 XT* __restrict__ z, size_t n) {
  for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < n; i += (size_t)gridDim.x * WG)
    z[i] = from_f32<XT>(siluf(g[i]) * u[i]);
}

// z = silu(g) * u, written as hi + lo bf16 parts for the matrix cores.
__global__ void __launch_bounds__(WG) k_silu_mul_split(const float* __restrict__ g, const float* __restrict__ u,
                                                       bf16* __restrict__ zh, bf16* __restrict__ zl, size_t n) {
  for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < n; i += (size_t)gridDim.x * WG) {
    const float z = siluf(g[i]) * u[i];
    const bf16 h = from_f32<bf16>(z);
    zh[i] = h;
    zl[i] = from_f32<bf16>(z - to_f32(h));
  }
}

__global__ void __launch_bounds__(WG) k_copy_f32(const float* __restrict__ src, float* __restrict__ dst,
                                                 float* __restrict__ dst2, int n) {
  for (int i = blockIdx.x * WG + threadIdx.x; i < n; i += gridDim.x * WG) {
    const float v = src[i];
    dst[i] = v;
    if (dst2) dst2[i] = v;
  }
}

// ---------------------------------------------------------------------------------------
// Causal GQA attention over the prompt on the matrix cores (bf16 cache, head_dim 64 or 128).
//
// Operands are prepared per layer by two small kernels: the rotated, pre-scaled queries are
// split as q = hi + lo (two bf16 parts, 16 significant bits); the keys the cache holds are
// gathered into a contiguous [T][Hkv*hd] copy and its values into a transposed one
// [Hkv*hd][Tp] (Tp = T padded to the key tile), so that every MFMA operand is a 16- or 8-byte
// contiguous load.  Attention reads exactly the values the cache stores (Section 4.3: decode
// later reads the same ones).
//
// One wave owns 32 query positions of one head and walks the key tiles (32 keys) up to its
// diagonal.  Everything is computed transposed, so that a lane owns ONE query column:
//   S^T[key][q] = K Q^T     (A = key rows, B = query columns; hi and lo parts of q)
//   O^T[dim][q] = V^T P^T   (A = rows of the transposed values, B = the probabilities straight
//                            from the accumulator registers of S^T, split hi + lo)
// The softmax statistics of a query are then per lane (plus one exchange with lane ^ 32), and
// rescaling O^T is a per-lane multiply.  Accumulator layout of the 32x32 MFMA: lane l holds
// column l % 32, register r holds row 8 (r / 4) + 4 (l / 32) + r % 4.
constexpr int FA_QW = 32;                 // queries per wave
constexpr int FA_KT = 32;                 // keys per tile

// q (fp32, rotated, scaled) -> hi / lo bf16.  grid-stride over n elements.
__global__ void __launch_bounds__(WG) k_split_bf16(const float* __restrict__ x, bf16* __restrict__ hi, bf16* __restrict__ lo, size_t n) {
  for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < n; i += (size_t)gridDim.x * WG) {
    const float v = x[i];
    const bf16 h = from_f32<bf16>(v);
    hi[i] = h;
    lo[i] = from_f32<bf16>(v - to_f32(h));
  }
}

// Cache pages -> kc[t][g*hd + d] and vt[(g*hd + d)][t] for 32 tokens of KV head g.
// grid = (ceil(T/32), Hkv); hd <= 128.
__global__ void __launch_bounds__(WG) k_kv_gather(const bf16* __restrict__ pool, size_t page_elems, const int* __restrict__ pt,
                                                  bf16* __restrict__ kc, bf16* __restrict__ vt, int T, int Tp, int Hkv,
                                                  int hd, int P) {
  __shared__ uint16_t vs[32][128 + 2];
  const int t0 = blockIdx.x * 32, g = blockIdx.y, nkv = Hkv * hd;
  const size_t head_off = (size_t)g * P * hd, v_off = (size_t)Hkv * P * hd;
  for (int i = threadIdx.x; i < 32 * hd; i += WG) {
    const int tt = i / hd, d = i - tt * hd, t = t0 + tt;
    uint16_t kvv = 0, vvv = 0;
    if (t < T) {
      const size_t base = (size_t)pt[t / P] * page_elems + head_off + (size_t)(t % P) * hd + d;
      kvv = pool[base].v;
      vvv = pool[base + v_off].v;
    }
    kc[(size_t)t * nkv + g * hd + d].v = kvv;                  // rows up to Tp exist
    vs[tt][d] = vvv;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 32 * hd; i += WG) {
    const int d = i / 32, tt = i - d * 32;
    vt[(size_t)(g * hd + d) * Tp + t0 + tt].v = vs[tt][d];
  }
}

// Output: hi + lo bf16 parts (outh, outl), the form the output projection consumes.
template <int HD>
__global__ void __launch_bounds__(WG) k_attn_flash(const bf16* __restrict__ qh, const bf16* __restrict__ ql,
                                                   const bf16* __restrict__ kc, const bf16* __restrict__ vt,
                                                   bf16* __restrict__ outh, bf16* __restrict__ outl, int T, int Tp, int Hq,
                                                   int Hkv) {
  constexpr int KS = HD / 16;             // k-steps of the score product
  constexpr int DT = HD / 32;             // 32-dim tiles of the output
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int col = lane & 31, gl = lane >> 5;
  const int h = blockIdx.y, g = h / (Hq / Hkv);
  const int q0 = (blockIdx.x * WAVES + wave) * FA_QW;
  if (q0 >= T) return;
  const int nq = Hq * HD, nkv = Hkv * HD;
  const int qi = q0 + col;                                       // this lane's query position
  const int qc = min(qi, T - 1);

  bf16x8_t Qh[KS], Ql[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    const size_t o = (size_t)qc * nq + h * HD + 16 * s + 8 * gl;
    Qh[s] = *reinterpret_cast<const bf16x8_t*>(qh + o);
    Ql[s] = *reinterpret_cast<const bf16x8_t*>(ql + o);
  }
  floatx16_t O[DT];
#pragma unroll
  for (int t = 0; t < DT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[t][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int n_tiles = (min(q0 + FA_QW, T) + FA_KT - 1) / FA_KT;  // keys 0 .. last query of the block
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int k0 = kt * FA_KT;
    // S^T = K Q^T
    floatx16_t S;
#pragma unroll
    for (int r = 0; r < 16; ++r) S[r] = 0.f;
    const bf16* krow = kc + (size_t)(k0 + col) * nkv + g * HD + 8 * gl;     // this lane's key row (A operand)
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(krow + 16 * s);
      S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, Ql[s], S, 0, 0, 0);
      S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, Qh[s], S, 0, 0, 0);
    }
    // causal mask and the tile's softmax statistics of this lane's query
    float mt = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = k0 + 8 * (r >> 2) + 4 * gl + (r & 3);
      if (key > qi) S[r] = -INFINITY;
      mt = fmaxf(mt, S[r]);
    }
    mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
    const float mn = fmaxf(m, mt);                 // finite: key 0 is visible to every query
    const float corr = __expf(m - mn);
    float ls = 0.f;
    floatx16_t Pv;
#pragma unroll
    for (int r = 0; r < 16; ++r) { Pv[r] = __expf(S[r] - mn); ls += Pv[r]; }
    ls += __shfl_xor(ls, 32, 64);
    l = l * corr + ls;
    m = mn;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[t][r] *= corr;
    // O^T += V^T P^T: k-step s2 uses accumulator registers 8 s2 .. 8 s2 + 7 of P as they are;
    // slot (gl, e) of that step is key k0 + 16 s2 + 8 (e / 4) + 4 gl + e % 4
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      bf16x8_t Ph, Pl;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float pv = Pv[8 * s2 + e];
        const bf16 hi = from_f32<bf16>(pv);
        const bf16 lo = from_f32<bf16>(pv - to_f32(hi));
        Ph[e] = __builtin_bit_cast(__bf16, hi.v);
        Pl[e] = __builtin_bit_cast(__bf16, lo.v);
      }
#pragma unroll
      for (int t = 0; t < DT; ++t) {
        const bf16* vrow = vt + (size_t)(g * HD + 32 * t + col) * Tp + k0 + 16 * s2 + 4 * gl;
        const uint2 v0 = *reinterpret_cast<const uint2*>(vrow);          // keys +0..3
        const uint2 v1 = *reinterpret_cast<const uint2*>(vrow + 8);      // keys +8..11
        union { uint4 u; bf16x8_t b; } vf;
        vf.u = make_uint4(v0.x, v0.y, v1.x, v1.y);
        O[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.b, Pl, O[t], 0, 0, 0);
        O[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.b, Ph, O[t], 0, 0, 0);
      }
    }
  }
  if (qi < T) {
    const float inv = 1.0f / l;
    const size_t orow = (size_t)qi * nq + h * HD;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float v = O[t][4 * rr + e] * inv;
          hi[e] = f2bf(v);
          lo[e] = f2bf(v - bf2f(hi[e]));
        }
        const size_t o = orow + 32 * t + 8 * rr + 4 * gl;
        *reinterpret_cast<uint2*>(outh + o) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
        *reinterpret_cast<uint2*>(outl + o) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
      }
  }
}

__global__ void k_set_int(int* p, int v) { if (threadIdx.x == 0 && blockIdx.x == 0) *p = v; }

__global__ void __launch_bounds__(WG) k_fill_u32(unsigned* p, unsigned v, size_t n) {
  for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < n; i += (size_t)gridDim.x * WG) p[i] = v;
}

// KV taps: positions [pos0, pos0+n) of one layer <-> dense fp32 [n][Hkv][hd].
template <typename KVT, bool WRITE>
__global__ void __launch_bounds__(WG) k_kv_tap(KVT* __restrict__ pool, size_t page_elems, const int* __restrict__ pt,
                                               int pos0, int Hkv, int hd, int P, float* __restrict__ kbuf,
                                               float* __restrict__ vbuf) {
  const int j = blockIdx.x, pos = pos0 + j;
  const size_t base = (size_t)pt[pos / P] * page_elems + (size_t)(pos % P) * hd;
  const size_t v_off = (size_t)Hkv * P * hd;
  for (int i = threadIdx.x; i < Hkv * hd; i += WG) {
    const int g = i / hd, d = i - g * hd;
    const size_t a = base + (size_t)g * P * hd + d;
    if (WRITE) {
      pool[a] = from_f32<KVT>(kbuf[(size_t)j * Hkv * hd + i]);
      pool[a + v_off] = from_f32<KVT>(vbuf[(size_t)j * Hkv * hd + i]);
    } else {
      kbuf[(size_t)j * Hkv * hd + i] = to_f32(pool[a]);
      vbuf[(size_t)j * Hkv * hd + i] = to_f32(pool[a + v_off]);
    }
  }
}

}  // namespace first
