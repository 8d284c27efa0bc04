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

// One workgroup's share of a batched attention launch: split `split` of `nsplit` of the sequence in slot `slot`,
// packed into one dword (slot | split << 8 | nsplit << 16) so that the kernel fetches it with a scalar load from its
// arguments (byte fields are fetched through the vector memory path: a full memory round trip before anything else).
typedef uint32_t AttnWork;
__host__ __device__ inline AttnWork attn_work_pack(int slot, int split, int nsplit) {
  return (uint32_t)slot | ((uint32_t)split << 8) | ((uint32_t)nsplit << 16);
}
constexpr int ATTN_WORK_MAX = 96;

struct BatchParams {
  DecParams d;          // geometry, per-sequence state, layer pointers (d.b unused)
  SeqList seqs;         // sequences of this pass; slot j <-> sequence seqs.id[j]
  bf16* xh;             // [BATCH_SLOTS * xpitch] high halves of the op's input vectors, A-operand order (bg_aidx)
  bf16* xl;             // low halves
  bf16* zh;             // MLP activation (written by gate/up, read by down), high halves, same order
  bf16* zl;             //                       low halves
  bf16* x2h;            // attention output (read by the output projection), high halves, same order
  bf16* x2l;            //                       low halves
  float* rinv;          // [BATCH_SLOTS] 1/rms of the vector that was split last (norm ops)
  // The output and down projections can leave the NEXT norm op's input behind (k_bgemv_g only): with fuse_gain set
  // their epilogue also writes the split of (updated h) * fuse_gain into xh / xl and, per tile group, the sum of
  // squares of its rows of h for every slot into ssq_part [group][BATCH_SLOTS].  The consumer is launched with
  // ssq_groups = that number of groups and forms 1/rms from the partial sums in a fixed order (bg_rinv_wave) instead of
  // reading rinv.  Producer and consumer must use the same slot list.
  const float* fuse_gain;
  float* ssq_part;
  int ssq_groups;
  SeqList next;         // with fuse_gain: slot list of the consuming norm op when it differs from seqs (next.n > 0); the
                        // epilogue then writes its rows of the split input and the sums of squares for those slots,
                        // reading back the residual rows it has just updated (and the untouched rows of the others)
  // k_attn_mfma_b with a work list (attn_nwork > 0): grid = (KV head, work item).  The host cuts every sequence into
  // splits in proportion to its length, so the workgroups of a batch of long and short sequences walk about the same
  // number of tiles and none is launched only to find that it has nothing to do.  Without a list: grid =
  // (split, KV head, slot), as many splits per sequence as the grid has.
  int attn_nwork;
  AttnWork attn_work[ATTN_WORK_MAX];
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
__device__ __forceinline__ bf16x8_t as_bf16x8(u32x4_t v) {
  union { u32x4_t u; bf16x8_t b; } c;
  c.u = v;
  return c.b;
}

// 1/rms of the norm op's input vectors (length K), one value per slot, computed by a whole wave: lane l ends up
// with the value of slot l / 4.  Either what k_xsplit stored, or formed from the producer's per-tile-group sums of
// squares: the four lanes of a slot take every fourth group each (eight loads in flight per lane), then the four
// sums are added in a fixed order - the same in every workgroup and launch.
__device__ __forceinline__ float bg_rinv_wave(const BatchParams& P, int K, int lane) {
  const int slot = lane >> 2, q = lane & 3;
  if (P.ssq_groups <= 0) return P.rinv[slot];
  float s = 0.f;
  for (int g0 = q; g0 < P.ssq_groups; g0 += 32) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int gi = g0 + 4 * u;
      v[u] = gi < P.ssq_groups ? P.ssq_part[gi * BATCH_SLOTS + slot] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  s += __shfl_xor(s, 1, 64);
  s += __shfl_xor(s, 2, 64);
  return 1.0f / sqrtf(s / (float)K + P.d.eps);
}

// hi/lo split of x (times gain) for slot blockIdx.x, elements [blockIdx.y * chunk, +chunk);
// rinv = 1/sqrt(mean(x^2) + eps) if gain (every workgroup of a slot sums the whole vector, the
// first one stores the result).  src: 0 = residual stream h, 1 = attention output.
__global__ void __launch_bounds__(WG) k_xsplit(BatchParams P, int src, int K, int chunk, const float* gain) {
  __shared__ float red[WAVES];
  const DecParams& p = P.d;
  const int j = blockIdx.x, b = P.seqs.id[j];
  const float* x = src == 0 ? p.h + (size_t)b * p.D : p.attn + (size_t)b * p.Hq * p.hd;
  bf16* xh = src == 0 ? P.xh : P.x2h;
  bf16* xl = src == 0 ? P.xl : P.x2l;
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
  SP.xh_out = P.x2h; SP.xl_out = P.x2l; SP.out_slot = blockIdx.z;
  sk_attention<HD, SK_WAVES, true>(SP, reinterpret_cast<bf16*>(p.kv_layer), S, blockIdx.y, blockIdx.x, nsplit, nullptr);
}

// Decode attention of (split, KV head, slot) for models with G = Hq / Hkv query heads per KV
// head (G = 4 instantiated): k_attn_tiles_b lets every head wave fetch its own copy of each
// 64-key tile and form scores and weighted values with scalar FMAs, which at long context is
// bound by the vector ALUs and by G-fold traffic through the compute unit's memory pipeline.
// Here a wave takes 16 keys (one cache page) at a time for ALL G heads and fetches them once,
// straight into the registers that use them (three pages per wave in flight; see Stage): scores
// = Q K^T on the matrix cores (16x16x32 bf16, Q split into high + low halves so that the product
// with the stored bf16 keys is exact to 2^-16), the G heads' online softmax side by side in the
// four 16-lane groups, weighted values with the value rows shared across the heads.  Between
// the prologue and the merge no wave waits for another.  The 8 waves' partial results meet in
// LDS; partial / count / merge across splits and the output format are those of
// sk_attention<.., SPLIT_OUT>.  The host sizes the grid to about one workgroup per compute unit.
// (An earlier version relayed 64-key tiles through 128 KB of LDS with a workgroup barrier per
// pair of tiles: 0.4 % slower steps at 16 k keys.)
constexpr int AS_THREADS = SK_WAVES * 64;
constexpr int AS_NT = 2;                                // fewest tiles the host gives a split
constexpr int AS_PT = 1024;                             // page ids of a split kept in LDS: the host gives a split at most AS_PT / 4 tiles
__host__ __device__ inline size_t as_lds_bytes(int G, int hd) {
  return ((size_t)G * hd + 2 * hd + hd + (size_t)SK_WAVES * G * (hd + 2) + 8 + AS_PT + SK_WAVES * (16 * 4 + 4)) * sizeof(float);
}

// Reductions over the 16 lanes of a DPP row (quads, half rows, rows): every lane ends up with
// the row's result, without LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_row_perm(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_row_perm<0xB1>(v)); v = fmaxf(v, dpp_row_perm<0x4E>(v));
  v = fmaxf(v, dpp_row_perm<0x141>(v)); v = fmaxf(v, dpp_row_perm<0x140>(v));
  return v;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_row_perm<0xB1>(v); v += dpp_row_perm<0x4E>(v);
  v += dpp_row_perm<0x141>(v); v += dpp_row_perm<0x140>(v);
  return v;
}

template <int HD, int G>
__global__ void __launch_bounds__(AS_THREADS) k_attn_mfma_b(BatchParams P) {
  static_assert(HD == 128 && G == 4, "lane layouts below: 8 value dims per lane, one head per group of four score rows");
  extern __shared__ __align__(16) float smem_f[];
  DecParams p = P.d;
  const bool listed = P.attn_nwork > 0;
  const AttnWork work = P.attn_work[listed ? blockIdx.y : 0];
  const int work_slot = work & 0xff, work_split = (work >> 8) & 0xff, work_nsplit = (work >> 16) & 0xff;
  const int slot = listed ? work_slot : (int)blockIdx.z;
  p.b = P.seqs.id[slot];
  constexpr int HALF = HD / 2;
  constexpr int KS = HD / 32;                           // MFMA k-steps over the head dimension
  constexpr int DL = HD / 16;                           // value dims per lane: lane (sub, dc), dc = lane % 16
  const int b = p.b, Pg = p.P, g = listed ? blockIdx.x : blockIdx.y;
  const int tid = threadIdx.x, wave = uni((int)(threadIdx.x >> 6)), lane = tid & 63;
  const int pos = uni(p.len[b]), nkeys = pos + 1, tiles = (nkeys + 63) >> 6;
  const int nsplit = max(1, min(listed ? work_nsplit : (int)gridDim.x, (tiles + AS_NT - 1) / AS_NT));
  const int s = listed ? work_split : (int)blockIdx.x;
  if (s >= nsplit) return;
  // LDS carve-up
  float* fb = smem_f;
  float* qs = fb; fb += G * HD;
  float* knew = fb; fb += HD;
  float* vnew = fb; fb += HD;
  float2* cs = reinterpret_cast<float2*>(fb); fb += HD;
  float* mbuf = fb; fb += SK_WAVES * G * (HD + 2);      // [wave][head][HD dims, max, sum]
  int* flag = reinterpret_cast<int*>(fb); fb += 8;
  int* pt_lds = reinterpret_cast<int*>(fb); fb += AS_PT;   // page ids of this split's slices: a lookup in global memory before every
                                                        // page request would put a second, dependent round trip in front of each
  float* wbuf = fb + (size_t)wave * (16 * 4 + 4);       // [16 keys][4 heads] softmax weights of this wave's slice, then the 4 heads' rescale factors
  const int tps = (tiles + nsplit - 1) / nsplit;
  const int t_first = s * tps, t_last = min(tiles, t_first + tps), T = max(0, t_last - t_first);
  // slices of 16 keys (one cache page each): wave w takes the split's slices w, w + 8, ...
  const int n_sl = max(0, min(4 * t_last, (nkeys + 15) >> 4) - 4 * t_first);
  const int nq = p.Hq * HD, nkv = p.Hkv * HD;
  const float* qkv = p.qkv + (size_t)b * (nq + 2 * nkv);
  const int* pt = p.page_table + (size_t)b * p.max_pages;
  bf16* pool = reinterpret_cast<bf16*>(p.kv_layer);
  const size_t head_off = (size_t)g * Pg * HD, v_off = (size_t)p.Hkv * Pg * HD;
  const bool owns_new = (pos >> 6) >= t_first && (pos >> 6) < t_last;
  const int last_page = pos / Pg;
  const int T1 = max(T, 1);                             // (a split without tiles still issues its requests, on a valid page)
  for (int i = tid; i < min(T1 * 4, AS_PT); i += AS_THREADS) pt_lds[i] = pt[min(t_first * 4 + i, last_page)];
  lds_barrier();

  // A slice's keys and values straight into the registers that use them: for the scores lane (key = lane % 16, kq = lane / 16)
  // holds dims 32 ks + 8 kq .. + 8 of its key (the B operand of MFMA k-step ks), for the weighted values lane (sub = lane / 16,
  // dc = lane % 16) holds dims 8 dc .. + 8 of keys 4 i + sub - sixteen 64-byte pieces per key request, four whole rows per
  // value request.  No wave needs another wave's keys, so nothing goes through LDS and the waves never wait for each other.
  struct Stage { u32x4_t k[KS], v[4]; };
  Stage st0, st1, st2;                                  // three slices of this wave in flight
  auto issue = [&](Stage& st, int j) __attribute__((always_inline)) {
    const int jj = max(0, min(j, n_sl - 1));             // (past the split: a harmless reload of a valid page)
    const int pg = pt_lds[min(jj, AS_PT - 1)];
    const bf16* base = pool + (size_t)pg * p.page_elems + head_off;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      st.k[ks] = *reinterpret_cast<const u32x4_t*>(base + (lane & 15) * HD + ks * 32 + ((lane >> 4) << 3));
#pragma unroll
    for (int i = 0; i < 4; ++i)
      st.v[i] = *reinterpret_cast<const u32x4_t*>(base + v_off + (4 * i + (lane >> 4)) * HD + (lane & 15) * DL);
  };

  // this step's q (G heads), k and v of the KV head (requested before the pages: loads return in order)
  {
    const int iq = min(tid, G * HALF - 1), hh = iq / HALF, dq = iq - hh * HALF;
    const int dk = min(tid, HALF - 1), dv = min(tid, HD - 1);
    const float q1 = qkv[(g * G + hh) * HD + dq], q2 = qkv[(g * G + hh) * HD + dq + HALF];
    const float k1 = qkv[nq + g * HD + dk], k2 = qkv[nq + g * HD + dk + HALF];
    const float vv = qkv[nq + nkv + g * HD + dv];
    const float2 c_own = p.rope_cs[(size_t)b * HALF + min(tid, HALF - 1)];               // made by k_embed_b
    issue(st0, wave);                                   // (a wave without slices reloads a valid page and ignores it)
    issue(st1, wave + SK_WAVES);
    issue(st2, wave + 2 * SK_WAVES);
    if (tid < HALF) cs[tid] = c_own;
    lds_barrier();
    if (tid < G * HALF) {                              // rotate and pre-scale the queries
      const float2 c = cs[dq];
      qs[hh * HD + dq] = (q1 * c.x - q2 * c.y) * p.qscale;
      qs[hh * HD + dq + HALF] = (q2 * c.x + q1 * c.y) * p.qscale;
    }
    if (owns_new) {                                    // append the new key / value; the rounded values also go to LDS
      const size_t base = (size_t)pt[pos / Pg] * p.page_elems + head_off + (size_t)(pos % Pg) * HD;
      if (tid < HALF) {
        const float2 c = cs[dk];
        const bf16 r1 = from_f32<bf16>(k1 * c.x - k2 * c.y), r2 = from_f32<bf16>(k2 * c.x + k1 * c.y);
        pool[base + dk] = r1; pool[base + dk + HALF] = r2;
        knew[dk] = __uint_as_float((unsigned)r1.v); knew[dk + HALF] = __uint_as_float((unsigned)r2.v);   // raw bf16 bits
      }
      if (tid < HD) {
        const bf16 r = from_f32<bf16>(vv);
        pool[base + v_off + dv] = r;
        vnew[dv] = __uint_as_float((unsigned)r.v);
      }
    }
  }
  lds_barrier();

  // A operand of the score MFMA: row m = lane % 16 holds query head m / 4, k = dims.  A lane's four result registers
  // are rows 4 (lane / 16) .. + 3, so the 16 lanes of group g = lane / 16 all hold the scores of head g (one key each):
  // the four heads' softmax steps run side by side in the four lane groups instead of one after the other in every lane.
  bf16x8_t qh[KS], ql[KS];
  {
    const int hm = (lane & 15) >> 2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      union { unsigned short u[8]; bf16x8_t v; } H, L;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = hm < G ? qs[hm * HD + ks * 32 + ((lane >> 4) << 3) + e] : 0.f;
        const bf16 h = from_f32<bf16>(x);
        H.u[e] = h.v; L.u[e] = from_f32<bf16>(x - to_f32(h)).v;
      }
      qh[ks] = H.v; ql[ks] = L.v;
    }
  }

  // per wave: running maximum, sum and weighted values of its 16-key slices, for all G heads;
  // lane (sub = lane / 16, dc = lane % 16) accumulates dims dc*DL .. +DL over keys 4 i + sub
  float m1 = -INFINITY, l1 = 0.f;                        // head lane / 16: running maximum and sum
  float o[G][DL];
#pragma unroll
  for (int h = 0; h < G; ++h) {
#pragma unroll
    for (int e = 0; e < DL; ++e) o[h][e] = 0.f;
  }
  const int sub = lane >> 4, dc = lane & 15;
  const int new_sl = (pos >> 4) - 4 * t_first;          // the slice that holds the new position (if this split owns it)

  auto slice = [&](Stage& st, int j) __attribute__((always_inline)) {
    if (j < n_sl) {
      const int k0 = (4 * t_first + j) << 4;             // first key of the slice
      if (owns_new && j == new_sl) {                     // the new position's row comes from this step, not from the cache
        const int r = pos & 15;
        if ((lane & 15) == r) {
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) {
            unsigned w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int d = ks * 32 + ((lane >> 4) << 3) + 2 * e;
              w[e] = (__float_as_uint(knew[d]) & 0xffffu) | (__float_as_uint(knew[d + 1]) << 16);
            }
            st.k[ks] = u32x4_t{w[0], w[1], w[2], w[3]};
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (4 * i + sub == r) {
            unsigned w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
              w[e] = (__float_as_uint(vnew[dc * DL + 2 * e]) & 0xffffu) | (__float_as_uint(vnew[dc * DL + 2 * e + 1]) << 16);
            st.v[i] = u32x4_t{w[0], w[1], w[2], w[3]};
          }
      }
      // scores: C[row = head][col = key]
      f32x4v_t sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8_t kb = as_bf16x8(st.k[ks]);
        sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qh[ks], kb, sc, 0, 0, 0);
        sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ql[ks], kb, sc, 0, 0, 0);
      }
      // lane (key = lane % 16, head = lane / 16): every register of sc is S[head][key]
      {
        const bool live = k0 + (lane & 15) < nkeys;
        const float sv = live ? sc[0] : -INFINITY;
        const float mt = row16_max(sv);
        const float mn = fmaxf(m1, mt);
        const float corr = mn == -INFINITY ? 1.f : expf(m1 - mn);        // (nothing seen yet)
        const float pv = live ? expf(sv - mn) : 0.f;
        const float ls = row16_sum(pv);
        l1 = l1 * corr + ls;
        m1 = mn;
        // the weights go through LDS: lane (sub, dc) needs those of keys 4 i + sub, for all heads
        wbuf[(lane & 15) * 4 + (lane >> 4)] = pv;
        if (__any(corr != 1.f)) {                          // (after the first slices the maxima rarely move: 1.0 would change nothing)
          if ((lane & 15) == 0) wbuf[64 + (lane >> 4)] = corr;
          const f32x4_t c4 = *reinterpret_cast<const f32x4_t*>(wbuf + 64);
#pragma unroll
          for (int h = 0; h < G; ++h)
#pragma unroll
            for (int e = 0; e < DL; ++e) o[h][e] *= c4[h];
        }
      }
      // weighted values: 4 rows per lane group, each value row shared by the G heads
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kr = 4 * i + sub;                      // key of this lane within the slice
        const int key = k0 + kr;
        const u32x4_t w = st.v[i];
        float vf[DL];
        vf[0] = __uint_as_float(w.x << 16); vf[1] = __uint_as_float(w.x & 0xffff0000u);
        vf[2] = __uint_as_float(w.y << 16); vf[3] = __uint_as_float(w.y & 0xffff0000u);
        vf[4] = __uint_as_float(w.z << 16); vf[5] = __uint_as_float(w.z & 0xffff0000u);
        vf[6] = __uint_as_float(w.w << 16); vf[7] = __uint_as_float(w.w & 0xffff0000u);
        if (k0 + 15 > pos) {                             // (only the slice that holds the last position has them)
#pragma unroll
          for (int e = 0; e < DL; ++e) vf[e] = key > pos ? 0.f : vf[e];        // never-written slots: no NaN patterns
        }
        const f32x4_t w4 = *reinterpret_cast<const f32x4_t*>(wbuf + kr * 4);   // weights of key kr for the G heads
#pragma unroll
        for (int h = 0; h < G; ++h) {
          const float wt = w4[h];
#pragma unroll
          for (int e = 0; e < DL; ++e) o[h][e] = fmaf(wt, vf[e], o[h][e]);
        }
      }
    }
    issue(st, j + 3 * SK_WAVES);
  };
  static_assert(DL == 8, "one 16-byte value load per lane and key");
  for (int j = wave; j < n_sl; j += 3 * SK_WAVES) {
    slice(st0, j);
    slice(st1, j + SK_WAVES);
    slice(st2, j + 2 * SK_WAVES);
  }

  // fold the key subgroups (lanes sub = 0..3), then every wave leaves its partial per head in LDS
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < DL; ++e) {
      o[h][e] += __shfl_xor(o[h][e], 16, 64);
      o[h][e] += __shfl_xor(o[h][e], 32, 64);
    }
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float* mb = mbuf + (size_t)(wave * G + h) * (HD + 2);
    if (lane < 16) {
#pragma unroll
      for (int e = 0; e < DL; ++e) mb[dc * DL + e] = o[h][e];
    }
  }
  if ((lane & 15) == 0) {
    float* mb = mbuf + (size_t)(wave * G + (lane >> 4)) * (HD + 2);
    mb[HD] = m1; mb[HD + 1] = l1;
  }
  __syncthreads();
  // wave h merges head h over the 8 waves (fixed order) and writes the split's partial
  if (wave < G) {
    const int hq = wave;
    float M = -INFINITY;
    for (int w2 = 0; w2 < SK_WAVES; ++w2) M = fmaxf(M, mbuf[(size_t)(w2 * G + hq) * (HD + 2) + HD]);
    float den = 0.f, a0 = 0.f, a1 = 0.f;
    for (int w2 = 0; w2 < SK_WAVES; ++w2) {
      const float* src = mbuf + (size_t)(w2 * G + hq) * (HD + 2);
      const float lt = src[HD + 1];
      if (lt > 0.f) {
        const float w = expf(src[HD] - M);
        den = fmaf(lt, w, den);
        a0 = fmaf(src[lane], w, a0);
        if (HD > 64) a1 = fmaf(src[lane + 64 < HD ? lane + 64 : lane], w, a1);
      }
    }
    const int H = g * G + hq;
    float* po = p.part_o + (((size_t)b * p.Hq + H) * S_MAX + s) * HD;
    st_coh(po + lane, a0);
    if (HD > 64) st_coh(po + lane + 64, a1);
    if (lane == 0) {
      float* pml = p.part_ml + (((size_t)b * p.Hq + H) * S_MAX + s) * 2;
      st_coh(pml, M); st_coh(pml + 1, den);
    }
  }
  // the last split of this KV head to finish merges all splits (fixed order) and writes the output
  vm_wait_all();
  __syncthreads();
  if (tid == 0) {
    const unsigned old = __hip_atomic_fetch_add(p.attn_cnt + b * p.Hkv + g, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (old == (unsigned)(nsplit - 1));
    if (last) __hip_atomic_store(p.attn_cnt + b * p.Hkv + g, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    flag[1] = last;
  }
  __syncthreads();
  if (uni(flag[1]) && wave < G) {
    constexpr int LPS = HD / 4, SPI = 64 / LPS, NI = 16;
    const int H = g * G + wave, q4 = (lane % LPS) * 4, sl = lane / LPS;
    const float* pml = p.part_ml + ((size_t)b * p.Hq + H) * S_MAX * 2;
    const float* po = p.part_o + ((size_t)b * p.Hq + H) * S_MAX * HD;
    float den = 0.f, M = -INFINITY;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    for (int b0 = 0; b0 < nsplit; b0 += NI * SPI) {
      f32x4_t o4[NI];
      float m_own, l_own;
#pragma unroll
      for (int i = 0; i < NI; ++i) coh_issue16(o4[i], po + min(b0 + i * SPI + sl, nsplit - 1) * HD + q4);
      coh_issue4(m_own, pml + 2 * min(lane, nsplit - 1));
      coh_issue4(l_own, pml + 2 * min(lane, nsplit - 1) + 1);
      coh_wait();
#pragma unroll
      for (int i = 0; i < NI; ++i) coh_use(o4[i]);
      coh_use(m_own); coh_use(l_own);
      float mv[NI], lv[NI];
      float Mb = M;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int ts = min(b0 + i * SPI + sl, nsplit - 1);
        mv[i] = __shfl(m_own, ts, 64); lv[i] = __shfl(l_own, ts, 64);
        if (b0 + i * SPI + sl < nsplit) Mb = fmaxf(Mb, mv[i]);
      }
#pragma unroll
      for (int off = LPS; off < 64; off <<= 1) Mb = fmaxf(Mb, __shfl_xor(Mb, off, 64));
      const float resc = expf(M - Mb);
      den *= resc; acc *= resc;
      M = Mb;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        if (b0 + i * SPI + sl < nsplit && lv[i] > 0.f) {
          const float w = expf(mv[i] - M);
          den = fmaf(lv[i], w, den);
          acc.x = fmaf(o4[i].x, w, acc.x); acc.y = fmaf(o4[i].y, w, acc.y);
          acc.z = fmaf(o4[i].z, w, acc.z); acc.w = fmaf(o4[i].w, w, acc.w);
        }
      }
    }
#pragma unroll
    for (int off = LPS; off < 64; off <<= 1) {
      den += __shfl_xor(den, off, 64);
      acc.x += __shfl_xor(acc.x, off, 64); acc.y += __shfl_xor(acc.y, off, 64);
      acc.z += __shfl_xor(acc.z, off, 64); acc.w += __shfl_xor(acc.w, off, 64);
    }
    if (sl == 0) {
      const float v[4] = {acc.x / den, acc.y / den, acc.z / den, acc.w / den};
      unsigned short hi[4], lo[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bf16 h = from_f32<bf16>(v[j]);
        hi[j] = h.v; lo[j] = from_f32<bf16>(v[j] - to_f32(h)).v;
      }
      const size_t at = bg_aidx(slot, H * HD + q4);
      *reinterpret_cast<uint2*>(P.x2h + at) = make_uint2(hi[0] | ((unsigned)hi[1] << 16), hi[2] | ((unsigned)hi[3] << 16));
      *reinterpret_cast<uint2*>(P.x2l + at) = make_uint2(lo[0] | ((unsigned)lo[1] << 16), lo[2] | ((unsigned)lo[3] << 16));
    }
  }
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
  const bf16* xh = (MODE == BG_DN ? P.zh : MODE == BG_O ? P.x2h : P.xh) + lane * 8;       // this lane's 16 bytes of block 0 (bg_aidx)
  const bf16* xl = (MODE == BG_DN ? P.zl : MODE == BG_O ? P.x2l : P.xl) + lane * 8;

  // norm ops: 1/rms of slot lane / 4 (requested here so that the loads overlap the weight stream)
  const float rv = (MODE == BG_QKV || MODE == BG_GU || MODE == BG_HEAD) ? bg_rinv_wave(P, K, lane) : 0.f;

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
  float rinv4[4];                                    // 1/rms of this lane's four slots (4 g + j)
#pragma unroll
  for (int j = 0; j < 4; ++j) rinv4[j] = __shfl(rv, (4 * g + j) * 4, 64);
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
        p.qkv[(size_t)b * N + row] = acc[t][j] * rinv4[j];
      } else if (MODE == BG_O || MODE == BG_DN) {
        p.h[(size_t)b * p.D + row] += acc[t][j];
      } else if (MODE == BG_GU) {
        const float r = rinv4[j];
        const float z = siluf(acc[2 * t][j] * r) * (acc[2 * t + 1][j] * r);
        const bf16 hi = from_f32<bf16>(z);
        P.zh[bg_aidx(slot, row)] = hi;                         // input of the down projection, already split
        P.zl[bg_aidx(slot, row)] = from_f32<bf16>(z - to_f32(hi));
      } else {
        P.logits_all[(size_t)b * N + row] = acc[t][j] * rinv4[j];
      }
    }
  }
}

// The mat-vecs of a layer decomposed the other way round: a workgroup = GW row tiles (one per wave) x
// ONE slice of K.  All its waves need the same slice of the activation operand, so it is copied into
// LDS once and read from there; k_bgemv's workgroup (tiles x slices of K over its waves) makes every
// wave fetch its own slice from L2, and that traffic counts against the same per-compute-unit memory
// pipeline as the weights (for the small matrices it is twice the weight bytes).  The K-slices of a
// tile group then live in different workgroups: each stores its partial sums, and the last one to
// finish (a counter per tile group) adds them in slice order - the result does not depend on which
// workgroup that is - and applies the epilogue.  GW (5..8 waves) and the number of slices are chosen
// on the host so that the workgroups come to a whole number of rounds over the compute units.
// Tile-order weights only.  Dynamic LDS: 2 * per * 1024 bytes (per = K-steps per slice).
__host__ __device__ inline int bgg_per(int K, int ks) { return (((K + 31) >> 5) + ks - 1) / ks; }

template <int MODE, int GW>
__global__ void __launch_bounds__(GW * 64) k_bgemv_g(BatchParams P, int N, int K, int ks, float* __restrict__ part,
                                                     unsigned* __restrict__ cnt) {
  static_assert(MODE == BG_QKV || MODE == BG_O || MODE == BG_DN || MODE == BG_GU, "the LM head has tiles enough for k_bgemv");
  constexpr int NS = MODE == BG_GU ? 2 : 1;            // gate/up: a wave streams the gate tile and the up tile of its rows
  constexpr int THREADS = GW * 64, ROWS = GW * 16;     // rows of a tile group
  extern __shared__ __align__(16) uint4 lds_a[];       // [hi, lo][per][64] 16-byte pieces in A-operand order
  __shared__ int last_flag;
  __shared__ float rinv_lds[BATCH_SLOTS];              // norm ops: 1/rms per slot
  const DecParams& p = P.d;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = lane & 15, g = lane >> 4;
  const int ksteps = (K + 31) >> 5, per = bgg_per(K, ks);
  const int tg = blockIdx.x / ks, sl = blockIdx.x % ks;
  const int s0 = sl * per, s1 = min(ksteps, s0 + per), ns = max(0, s1 - s0);
  const int ntiles = (N + 15) >> 4, tile = tg * GW + wave;
  const bf16* w[NS];
#pragma unroll
  for (int i = 0; i < NS; ++i) w[i] = bg_tiled_base<MODE>(P, i) + (size_t)min(tile, ntiles - 1) * ksteps * 512 + lane * 8;

  constexpr int UN = 4;
  struct Chunk { uint4 wv[UN][NS]; };
  const int nchunks = ns / UN;
  auto load = [&](Chunk& c, int ci) __attribute__((always_inline)) {
    const int sc = s0 + min(ci, max(nchunks - 1, 0)) * UN;
#pragma unroll
    for (int u = 0; u < UN; ++u)
#pragma unroll
      for (int i = 0; i < NS; ++i) c.wv[u][i] = ld_stream16(w[i] + (size_t)min(sc + u, ksteps - 1) * 512);
  };
  Chunk A, B;
  load(A, 0);                                          // the weight stream starts before the activations are staged
  {
    const uint4* xh = reinterpret_cast<const uint4*>((MODE == BG_DN ? P.zh : MODE == BG_O ? P.x2h : P.xh) + (size_t)s0 * 512);
    const uint4* xl = reinterpret_cast<const uint4*>((MODE == BG_DN ? P.zl : MODE == BG_O ? P.x2l : P.xl) + (size_t)s0 * 512);
    // A thread's pieces are requested in runs of 8, 4, 2 and 1 - every load of a run before its first write to LDS -
    // so staging costs a few memory round trips (behind the weight loads already in flight), not one per piece.
    const int np = ns * 64;
    auto run = [&](int i0, auto sbc) __attribute__((always_inline)) {
      constexpr int SB = decltype(sbc)::value;
      u32x4_t vh[SB], vl[SB];
#pragma unroll
      for (int u = 0; u < SB; ++u) {
        vh[u] = *reinterpret_cast<const u32x4_t*>(xh + i0 + u * THREADS);
        vl[u] = *reinterpret_cast<const u32x4_t*>(xl + i0 + u * THREADS);
      }
#pragma unroll
      for (int u = 0; u < SB; ++u) {
        *reinterpret_cast<u32x4_t*>(lds_a + i0 + u * THREADS) = vh[u];
        *reinterpret_cast<u32x4_t*>(lds_a + per * 64 + i0 + u * THREADS) = vl[u];
      }
    };
    int i0 = tid;
    for (; i0 + 7 * THREADS < np; i0 += 8 * THREADS) run(i0, std::integral_constant<int, 8>{});
    if (i0 + 3 * THREADS < np) { run(i0, std::integral_constant<int, 4>{}); i0 += 4 * THREADS; }
    if (i0 + THREADS < np) { run(i0, std::integral_constant<int, 2>{}); i0 += 2 * THREADS; }
    if (i0 < np) run(i0, std::integral_constant<int, 1>{});
  }
  if ((MODE == BG_QKV || MODE == BG_GU) && wave == 0) {
    const float rv = bg_rinv_wave(P, K, lane);
    if ((lane & 3) == 0) rinv_lds[lane >> 2] = rv;
  }
  __syncthreads();

  f32x4v_t acc[NS];
#pragma unroll
  for (int i = 0; i < NS; ++i) acc[i] = f32x4v_t{0.f, 0.f, 0.f, 0.f};
  auto mma = [&](const Chunk& c, int ci) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const bf16x8_t ah = as_bf16x8(lds_a[(ci * UN + u) * 64 + lane]);
      const bf16x8_t al = as_bf16x8(lds_a[per * 64 + (ci * UN + u) * 64 + lane]);
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const bf16x8_t bw = as_bf16x8(c.wv[u][i]);
        acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bw, acc[i], 0, 0, 0);
        acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bw, acc[i], 0, 0, 0);
      }
    }
  };
  if (nchunks > 0) {
    int ci = 0;
    for (; ci + 2 <= nchunks; ci += 2) {
      load(B, ci + 1);
      mma(A, ci);
      load(A, ci + 2);
      mma(B, ci + 1);
    }
    if (ci < nchunks) mma(A, ci);
  }
  for (int s = s0 + nchunks * UN; s < s1; ++s) {       // remaining steps of the slice
    const bf16x8_t ah = as_bf16x8(lds_a[(s - s0) * 64 + lane]), al = as_bf16x8(lds_a[per * 64 + (s - s0) * 64 + lane]);
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      const bf16x8_t bw = as_bf16x8(*reinterpret_cast<const uint4*>(w[i] + (size_t)s * 512));
      acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bw, acc[i], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bw, acc[i], 0, 0, 0);
    }
  }

  // partial sums of this slice: [workgroup][stream][slot][row within the tile group]
  float* mine = part + (size_t)blockIdx.x * (NS * 16 * ROWS);
#pragma unroll
  for (int i = 0; i < NS; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) st_coh(mine + i * (16 * ROWS) + (4 * g + j) * ROWS + wave * 16 + n, acc[i][j]);
  vm_wait_all();
  __syncthreads();
  if (tid == 0) {
    const unsigned old = __hip_atomic_fetch_add(cnt + tg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = old == (unsigned)(ks - 1);
    if (last) __hip_atomic_store(cnt + tg, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last_flag = last;
  }
  __syncthreads();
  if (!last_flag) return;
  // the last slice of this tile group to finish adds the slices in order and applies the epilogue
  const float* grp = part + (size_t)tg * ks * (NS * 16 * ROWS);
  __shared__ float ssq_lds[(MODE == BG_O || MODE == BG_DN) ? BATCH_SLOTS * ROWS : 1];   // squares of the updated h, [slot][row]
  const bool fuse = (MODE == BG_O || MODE == BG_DN) && P.fuse_gain != nullptr;
  const bool remap = fuse && P.next.n > 0;
  auto finish = [&](int e, const float (&sum)[NS]) __attribute__((always_inline)) {
    const int slot = e / ROWS, r = e % ROWS, row = tg * ROWS + r;
    if (slot >= P.seqs.n || row >= N) {
      if (MODE == BG_O || MODE == BG_DN) ssq_lds[e] = 0.f;
      return;
    }
    const int b = P.seqs.id[slot];
    if (MODE == BG_QKV) {
      p.qkv[(size_t)b * N + row] = sum[0] * rinv_lds[slot];
    } else if (MODE == BG_GU) {
      const float rr = rinv_lds[slot];
      const float z = siluf(sum[0] * rr) * (sum[NS - 1] * rr);
      const bf16 hi = from_f32<bf16>(z);
      P.zh[bg_aidx(slot, row)] = hi;                           // input of the down projection, already split
      P.zl[bg_aidx(slot, row)] = from_f32<bf16>(z - to_f32(hi));
    } else {
      const float hn = p.h[(size_t)b * p.D + row] + sum[0];
      p.h[(size_t)b * p.D + row] = hn;
      ssq_lds[e] = hn * hn;
      if (fuse && !remap) {                                    // the next norm op's input, split as k_xsplit would
        const float v = hn * P.fuse_gain[row];
        const bf16 hi = from_f32<bf16>(v);
        P.xh[bg_aidx(slot, row)] = hi;
        P.xl[bg_aidx(slot, row)] = from_f32<bf16>(v - to_f32(hi));
      }
    }
  };
  if constexpr (MODE == BG_QKV || MODE == BG_GU) {
    // every partial sum this thread needs - its 4 elements x streams x up to 8 slices - is requested before the first
    // is used: one memory round trip for the whole epilogue instead of one per element and stream
    constexpr int EPT = 16 * ROWS / THREADS;
    static_assert(EPT * THREADS == 16 * ROWS, "whole rounds");
    float pv[EPT][NS][8];
#pragma unroll
    for (int u = 0; u < EPT; ++u)
#pragma unroll
      for (int i = 0; i < NS; ++i)
#pragma unroll
        for (int q = 0; q < 8; ++q)
          coh_issue4(pv[u][i][q], grp + (size_t)min(q, ks - 1) * (NS * 16 * ROWS) + i * (16 * ROWS) + tid + u * THREADS);
    coh_wait();
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
      float sum[NS];
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        sum[i] = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) { coh_use(pv[u][i][q]); if (q < ks) sum[i] += pv[u][i][q]; }
      }
      finish(tid + u * THREADS, sum);
    }
  } else {
    // (the projections that add to the residual stream take one element per round: measured, the batch of loads
    //  above makes them slower)
    for (int e = tid; e < 16 * ROWS; e += THREADS) {
      float sum[NS];
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        float v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) coh_issue4(v[q], grp + (size_t)min(q, ks - 1) * (NS * 16 * ROWS) + i * (16 * ROWS) + e);
        coh_wait();
        sum[i] = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) { coh_use(v[q]); if (q < ks) sum[i] += v[q]; }
      }
      finish(e, sum);
    }
  }
  if ((MODE == BG_O || MODE == BG_DN) && remap) {
    // the consumer's slots: this group's rows of every sequence it will read, straight from the residual stream
    __syncthreads();                                           // (waits for the stores above as well)
    constexpr int PER = 16 * ROWS / THREADS;                   // elements per thread
    static_assert(PER * THREADS == 16 * ROWS, "whole rounds");
    float hv[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int e = tid + u * THREADS, slot = e / ROWS, row = tg * ROWS + e % ROWS;
      const bool ok = slot < P.next.n && row < N;
      hv[u] = p.h[(size_t)P.next.id[ok ? slot : 0] * p.D + (ok ? row : 0)];   // (rows stored above: same workgroup, after the barrier)
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int e = tid + u * THREADS, slot = e / ROWS, row = tg * ROWS + e % ROWS;
      const bool ok = slot < P.next.n && row < N;
      ssq_lds[e] = ok ? hv[u] * hv[u] : 0.f;
      if (ok) {
        const float v = hv[u] * P.fuse_gain[row];
        const bf16 hi = from_f32<bf16>(v);
        P.xh[bg_aidx(slot, row)] = hi;
        P.xl[bg_aidx(slot, row)] = from_f32<bf16>(v - to_f32(hi));
      }
    }
  }
  if ((MODE == BG_O || MODE == BG_DN) && fuse) {
    __syncthreads();
    if (tid < 64) {                                            // four lanes per slot, a quarter of the group's rows each, fixed order
      const int sl2 = tid >> 2, qd = tid & 3;
      float q = 0.f;
      for (int r = qd * (ROWS / 4); r < (qd + 1) * (ROWS / 4); ++r) q += ssq_lds[sl2 * ROWS + r];
      q += __shfl_xor(q, 1, 64);
      q += __shfl_xor(q, 2, 64);
      if (qd == 0) P.ssq_part[tg * BATCH_SLOTS + sl2] = q;
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
