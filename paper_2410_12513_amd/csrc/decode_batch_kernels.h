// Decode step of a BATCH of sequences with per-sequence skip masks (Section 4.3 item 2 with
// the batch sizes of Section 5's latency tables).  For each layer the host forms the list of
// sequences that keep it; the layer's weights are then streamed from HBM ONCE for the whole
// list: every mat-vec becomes a skinny matrix product  Y[seq][row] = sum_k W[row][k] X[seq][k]
// with up to 16 sequences, which is one MFMA tile wide.
//
// Activations stay fp32 between ops.  For the matrix cores each activation vector is split
// as x = hi + lo with hi = bf16(x), lo = bf16(x - hi) (16 significant bits), and every weight
// tile is multiplied with both halves, accumulating in fp32.  RMSNorm's gain is applied before
// the split and its 1/rms after the product (it is one scalar per sequence).
#pragma once
#include "decode_kernels.h"
#include "step_kernel.h"

namespace first {

constexpr int BATCH_SLOTS = 16;      // sequences per pass = rows of one MFMA tile
constexpr int BG_THREADS = 512;      // 8 waves: (row tiles per workgroup) x (slices of K) = 8
constexpr int BG_WAVES = BG_THREADS / 64;

struct SeqList {
  int n;
  int id[BATCH_SLOTS];
};

struct BatchParams {
  DecParams d;          // geometry, per-sequence state, layer pointers (d.b unused)
  SeqList seqs;         // sequences of this pass; slot j <-> sequence seqs.id[j]
  bf16* xh;             // [BATCH_SLOTS * xpitch] high halves of the op's input vectors, A-operand order (bg_aidx)
  bf16* xl;             // low halves
  bf16* zh;             // MLP activation (written by gate/up, read by down), high halves, same order
  bf16* zl;             //                       low halves
  float* rinv;          // [BATCH_SLOTS] 1/rms of the vector that was split last (norm ops)
  int xpitch;
  float* logits_all;    // [B][V] logits of the step (caller's buffer or the library's)
  // optional copies of the layer's matrices (and of the LM head) in MFMA tile order, see k_tile_weights
  const bf16 *t_qkv, *t_o, *t_g, *t_u, *t_d, *t_head;
};

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4v_t;

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8_t b; } c;
  c.u = v;
  return c.b;
}

// hi/lo split of x (times gain) for slot blockIdx.x, elements [blockIdx.y * chunk, +chunk);
// rinv = 1/sqrt(mean(x^2) + eps) if gain (every workgroup of a slot sums the whole vector, the
// first one stores the result).  src: 0 = residual stream h, 1 = attention output.
__global__ void __launch_bounds__(WG) k_xsplit(BatchParams P, int src, int K, int chunk, const float* gain) {
  __shared__ float red[WAVES];
  const DecParams& p = P.d;
  const int j = blockIdx.x, b = P.seqs.id[j];
  const float* x = src == 0 ? p.h + (size_t)b * p.D : p.attn + (size_t)b * p.Hq * p.hd;
  bf16* xh = P.xh;
  bf16* xl = P.xl;
  if (gain && blockIdx.y == 0) {
    float ss = 0.f;
    for (int k = threadIdx.x; k < K; k += WG) { const float v = x[k]; ss = fmaf(v, v, ss); }
    const float tot = block_sum(ss, red);
    if (threadIdx.x == 0) P.rinv[j] = 1.0f / sqrtf(tot / (float)K + p.eps);
  }
  const int k0 = blockIdx.y * chunk, k1 = min(K, k0 + chunk);
  for (int k = k0 + threadIdx.x; k < k1; k += WG) {
    float v = x[k];
    if (gain) v *= gain[k];
    const bf16 hi = from_f32<bf16>(v);
    xh[bg_aidx(j, k)] = hi;
    xl[bg_aidx(j, k)] = from_f32<bf16>(v - to_f32(hi));
  }
}

// h = E[token] and the rotation table of the position, for slot blockIdx.x.
__global__ void __launch_bounds__(WG) k_embed_b(BatchParams P) {
  DecParams p = P.d;
  p.b = P.seqs.id[blockIdx.x];
  phase_embed<bf16>(p);
}

// Decode attention of (split, KV head, slot).
__global__ void __launch_bounds__(WG) k_attn_b(BatchParams P) {
  extern __shared__ __align__(16) char smem_raw[];
  DecParams p = P.d;
  p.b = P.seqs.id[blockIdx.z];
  phase_attn<bf16>(p, blockIdx.y, blockIdx.x, smem_raw);
}

// Decode attention of (split, KV head, slot) with the persistent kernel's attention phase
// (register-resident 64-key tiles, page lookups batched per tile): SK_WAVES worker waves (query
// heads x key groups).  A workgroup's life is a chain of memory round trips (q/k/v, key tile,
// value tile, partial, count, merge), so two workgroups share a compute unit (at most 128
// registers per lane).  Needs 16-token pages and G <= SK_WAVES.
constexpr int AT_THREADS = SK_WAVES * 64;
template <int HD>
__global__ void __launch_bounds__(AT_THREADS, 4) k_attn_tiles_b(BatchParams P) {
  extern __shared__ __align__(16) float smem_f[];
  StepParams SP{};
  SP.d = P.d;
  SP.d.b = P.seqs.id[blockIdx.z];
  const DecParams& p = SP.d;
  const SkLds S = sk_carve(smem_f, 0, 0, 0, p.G, HD);
  const int tid = threadIdx.x;
  const int pos = uni(p.len[p.b]);
  // The grid is sized for the longest sequence; a shorter one uses only as many splits as give
  // every worker wave a 64-key tile, and the workgroups of its other splits leave at once.
  const int tiles = (pos + 64) >> 6, nkg = max(1, SK_WAVES / p.G);
  const int nsplit = max(1, min((int)gridDim.x, (tiles + nkg - 1) / nkg));
  if ((int)blockIdx.x >= nsplit) return;
  for (int i = tid; i < HD / 2; i += AT_THREADS) S.cs[i] = p.rope_cs[(size_t)p.b * (HD / 2) + i];   // made by k_embed_b
  lds_barrier();
  // the merged output goes out split into bf16 high and low halves, in the order the output
  // projection's A operand reads (slot = position of the sequence in this pass)
  SP.xh_out = P.xh; SP.xl_out = P.xl; SP.out_slot = blockIdx.z;
  sk_attention<HD, SK_WAVES, false, true>(SP, reinterpret_cast<bf16*>(p.kv_layer), S, blockIdx.y, blockIdx.x, nsplit, nullptr);
}

// Re-lays a row-major bf16 matrix W[N][K] into MFMA tile order: block (t, s) = rows 16 t .. +16,
// columns 32 s .. +32 is 1 KB, lane l of a wave owns its 16 bytes l (row 16 t + l % 16, columns
// 32 s + 8 (l / 16) .. +8), blocks of a tile are consecutive in s.  A wave then streams a tile
// as contiguous 1 KB loads instead of sixteen 64-byte pieces 2 K bytes apart, which measured
// 1.3-1.6x faster for the batched mat-vecs.  Rows past N and columns past K are zero.
__global__ void __launch_bounds__(WG) k_tile_weights(const bf16* __restrict__ src, bf16* __restrict__ dst, int N, int K) {
  const int ksteps = (K + 31) >> 5, tiles = (N + 15) >> 4;
  const size_t total = (size_t)tiles * ksteps * 64;
  for (size_t idx = (size_t)blockIdx.x * WG + threadIdx.x; idx < total; idx += (size_t)gridDim.x * WG) {
    const size_t blk = idx >> 6;
    const int l = (int)(idx & 63), t = (int)(blk / ksteps), sblk = (int)(blk - (size_t)t * ksteps);
    const int row = 16 * t + (l & 15), k = 32 * sblk + 8 * (l >> 4);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < N && k < K) v = *reinterpret_cast<const uint4*>(src + (size_t)row * K + k);
    *reinterpret_cast<uint4*>(dst + idx * 8) = v;
  }
}

enum { BG_QKV = 0, BG_O = 1, BG_GU = 2, BG_DN = 3, BG_HEAD = 4 };

// Y[slot][row] for RT tiles of 16 rows per wave group.  Workgroup = 8 waves = (8 / kslices) tile
// groups x kslices slices of the contraction; the slices of a group are added in slice order
// in LDS, so results do not depend on timing.  The RT tiles of a wave share its activation
// operands (the activations come from L2 for every tile group, so RT divides that traffic).
//
// MFMA 16x16x32 operands: A = activations (rows = slots, lane l: slot l % 16, k = 8 (l / 16) ..+8),
// B = weights (columns = weight rows, lane l: row l % 16, same k), C: lane l holds weight row
// l % 16 for slots 4 (l / 16) .. +4.
template <int MODE>
__device__ __forceinline__ const bf16* bg_row_ptr(const DecParams& p, int rowc, int K, int which) {
  if (MODE == BG_QKV) {
    const int nq = p.Hq * p.hd, nk = p.Hkv * p.hd;
    return rowc < nq ? reinterpret_cast<const bf16*>(p.wq) + (size_t)rowc * K
         : rowc < nq + nk ? reinterpret_cast<const bf16*>(p.wk) + (size_t)(rowc - nq) * K
                          : reinterpret_cast<const bf16*>(p.wv) + (size_t)(rowc - nq - nk) * K;
  }
  if (MODE == BG_O) return reinterpret_cast<const bf16*>(p.wo) + (size_t)rowc * K;
  if (MODE == BG_GU) return reinterpret_cast<const bf16*>(which ? p.wu : p.wg) + (size_t)rowc * K;
  if (MODE == BG_DN) return reinterpret_cast<const bf16*>(p.wd) + (size_t)rowc * K;
  return reinterpret_cast<const bf16*>(p.lm_head) + (size_t)rowc * K;
}

template <int MODE>
__device__ __forceinline__ const bf16* bg_tiled_base(const BatchParams& P, int which) {
  return MODE == BG_QKV ? P.t_qkv : MODE == BG_O ? P.t_o : MODE == BG_GU ? (which ? P.t_u : P.t_g)
       : MODE == BG_DN ? P.t_d : P.t_head;
}

// TILED: the weights come from the tile-order copies (every load of a wave is 1 KB contiguous,
// zero padding instead of a ragged last step); otherwise from the caller's row-major matrices.
template <int MODE, int RT, bool TILED>
__global__ void __launch_bounds__(BG_THREADS) k_bgemv(BatchParams P, int N, int K, int kslices) {
  constexpr int NS = MODE == BG_GU ? 2 * RT : RT;   // weight streams per wave (gate and up rows of a tile are two)
  __shared__ float red[BG_WAVES][NS][4][64];
  const DecParams& p = P.d;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = lane & 15, g = lane >> 4;
  const int groups_per_wg = BG_WAVES / kslices;
  const int group = blockIdx.x * groups_per_wg + wave / kslices, slice = wave % kslices;
  const int ksteps = (K + 31) >> 5;
  const int per = (ksteps + kslices - 1) / kslices;
  const int s0 = slice * per, s1 = min(ksteps, s0 + per);

  const bf16* w[NS];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    if (TILED) {
      // stream pointer = this lane's 16 bytes of block (tile, step 0); a step advances it by 512 elements
      const int tile = min(group * RT + t, ((N + 15) >> 4) - 1);
      const size_t off = (size_t)tile * ksteps * 512 + lane * 8;
      if (MODE == BG_GU) { w[2 * t] = bg_tiled_base<MODE>(P, 0) + off; w[2 * t + 1] = bg_tiled_base<MODE>(P, 1) + off; }
      else w[t] = bg_tiled_base<MODE>(P, 0) + off;
    } else {
      const int rowc = min((group * RT + t) * 16 + n, N - 1);
      if (MODE == BG_GU) { w[2 * t] = bg_row_ptr<MODE>(p, rowc, K, 0); w[2 * t + 1] = bg_row_ptr<MODE>(p, rowc, K, 1); }
      else w[t] = bg_row_ptr<MODE>(p, rowc, K, 0);
    }
  }
  const bf16* xh = (MODE == BG_DN ? P.zh : P.xh) + lane * 8;       // this lane's 16 bytes of block 0 (bg_aidx)
  const bf16* xl = (MODE == BG_DN ? P.zl : P.xl) + lane * 8;

  f32x4v_t acc[NS];
#pragma unroll
  for (int i = 0; i < NS; ++i) acc[i] = f32x4v_t{0.f, 0.f, 0.f, 0.f};
  const int full1 = TILED ? s1 : min(s1, K >> 5);  // steps in which every lane's 8 elements are in range (tiles are zero-padded)
  int s = s0;
  // Main loop over chunks of UN k-steps, software-pipelined: the loads of the next chunk are in
  // flight while the matrix cores work on the current one (two register sets, alternating).
  // Branch-free: a chunk index past the end is clamped to the last chunk (a harmless re-load),
  // so the compiler keeps exact counts of the loads in flight.
  constexpr int UN = NS >= 4 ? 2 : 4;              // k-steps per chunk
  struct Chunk { uint4 a_h[UN], a_l[UN], wv[UN][NS]; };
  const int nchunks = max(0, (full1 - s0) / UN);
  auto load = [&](Chunk& c, int ci) {
    const int sc = s0 + min(ci, nchunks - 1) * UN;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int k = ((sc + u) << 5) + (g << 3);
#pragma unroll
      for (int i = 0; i < NS; ++i) c.wv[u][i] = ld_stream16(TILED ? w[i] + (size_t)(sc + u) * 512 : w[i] + k);
      c.a_h[u] = *reinterpret_cast<const uint4*>(xh + ((size_t)(sc + u) << 9));
      c.a_l[u] = *reinterpret_cast<const uint4*>(xl + ((size_t)(sc + u) << 9));
    }
  };
  auto mma = [&](const Chunk& c) {
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const bf16x8_t ah = as_bf16x8(c.a_h[u]), al = as_bf16x8(c.a_l[u]);
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const bf16x8_t bw = as_bf16x8(c.wv[u][i]);
        acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bw, acc[i], 0, 0, 0);
        acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bw, acc[i], 0, 0, 0);
      }
    }
  };
  if (nchunks > 0) {
    Chunk A, B;
    load(A, 0);
    int ci = 0;
    for (; ci + 2 <= nchunks; ci += 2) {
      load(B, ci + 1);
      mma(A);
      load(A, ci + 2);
      mma(B);
    }
    if (ci < nchunks) mma(A);                      // odd count: the last chunk is already in A
    s = s0 + nchunks * UN;
  }
  for (; s < s1; ++s) {                            // remaining steps; the last may be ragged (K a multiple of 8, not of 32)
    const int k = (s << 5) + (g << 3);
    uint4 ah4 = make_uint4(0, 0, 0, 0), al4 = ah4, wv[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) wv[i] = ah4;
    if (k < K) {
      ah4 = *reinterpret_cast<const uint4*>(xh + ((size_t)s << 9));
      al4 = *reinterpret_cast<const uint4*>(xl + ((size_t)s << 9));
#pragma unroll
      for (int i = 0; i < NS; ++i) wv[i] = *reinterpret_cast<const uint4*>(TILED ? w[i] + (size_t)s * 512 : w[i] + k);
    }
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ah4), as_bf16x8(wv[i]), acc[i], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(al4), as_bf16x8(wv[i]), acc[i], 0, 0, 0);
    }
  }

  if (kslices > 1) {
#pragma unroll
    for (int i = 0; i < NS; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) red[wave][i][j][lane] = acc[i][j];
    __syncthreads();
    if (slice != 0) return;
#pragma unroll
    for (int i = 0; i < NS; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float a = red[wave][i][j][lane];
        for (int t = 1; t < kslices; ++t) a += red[wave + t][i][j][lane];
        acc[i][j] = a;
      }
  }
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const int row = (group * RT + t) * 16 + n;
    if (row >= N) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int slot = 4 * g + j;
      if (slot >= P.seqs.n) continue;
      const int b = P.seqs.id[slot];
      if (MODE == BG_QKV) {
        p.qkv[(size_t)b * N + row] = acc[t][j] * P.rinv[slot];
      } else if (MODE == BG_O || MODE == BG_DN) {
        p.h[(size_t)b * p.D + row] += acc[t][j];
      } else if (MODE == BG_GU) {
        const float r = P.rinv[slot];
        const float z = siluf(acc[2 * t][j] * r) * (acc[2 * t + 1][j] * r);
        const bf16 hi = from_f32<bf16>(z);
        P.zh[bg_aidx(slot, row)] = hi;                         // input of the down projection, already split
        P.zl[bg_aidx(slot, row)] = from_f32<bf16>(z - to_f32(hi));
      } else {
        P.logits_all[(size_t)b * N + row] = acc[t][j] * P.rinv[slot];
      }
    }
  }
}

// Greedy token, stage 1: candidate of chunk blockIdx.y of slot blockIdx.x's logits row.
constexpr int ARG_CHUNKS = 64;
__global__ void __launch_bounds__(WG) k_argmax_part_b(BatchParams P) {
  __shared__ Best wbest[WAVES];
  const DecParams& p = P.d;
  const int b = P.seqs.id[blockIdx.x], tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* lg = P.logits_all + (size_t)b * p.V;
  const int per = (p.V + ARG_CHUNKS - 1) / ARG_CHUNKS, r0 = blockIdx.y * per, r1 = min(p.V, r0 + per);
  Best best{-INFINITY, 0x7fffffff};
  for (int r = r0 + tid; r < r1; r += WG) {
    const Best c{lg[r], r};
    if (better(c, best)) best = c;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const Best c{__shfl_xor(best.v, o, 64), __shfl_xor(best.i, o, 64)};
    if (better(c, best)) best = c;
  }
  if (lane == 0) wbest[wave] = best;
  __syncthreads();
  if (tid == 0) {
    for (int wv = 1; wv < WAVES; ++wv)
      if (better(wbest[wv], best)) best = wbest[wv];
    p.arg_part[(size_t)b * ARG_MAX_WG + blockIdx.y] = best;
  }
}

// Stage 2: lowest index among the best candidates; advances the sequence length.
__global__ void __launch_bounds__(64) k_argmax_final_b(BatchParams P, int advance) {
  const DecParams& p = P.d;
  const int b = P.seqs.id[blockIdx.x], lane = threadIdx.x;
  Best best = lane < ARG_CHUNKS ? p.arg_part[(size_t)b * ARG_MAX_WG + lane] : Best{-INFINITY, 0x7fffffff};
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const Best c{__shfl_xor(best.v, o, 64), __shfl_xor(best.i, o, 64)};
    if (better(c, best)) best = c;
  }
  if (lane == 0) {
    if (p.token_out) p.token_out[b] = best.i;
    if (advance) p.len[b] += 1;
  }
}

}  // namespace first
