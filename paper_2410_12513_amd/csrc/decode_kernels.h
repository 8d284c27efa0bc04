// Decode-step kernels: one token per sequence through the kept layers (Section 4.3 item 2).
// Every phase is a __device__ function of (workgroup index, workgroup count) so that the
// same code serves the one-kernel-per-op launches and the persistent whole-step kernel.
#pragma once
#include "common.h"

namespace first {

// Everything a decode phase needs.  Passed by value as the kernel argument.
struct DecParams {
  // geometry
  int D, Hq, Hkv, hd, F, V, G;       // G = Hq / Hkv
  int P, max_pages;                  // KV page size in tokens, page-table row length
  int S;                             // KV splits per (sequence, KV head) in attention
  float eps, qscale;                 // RMSNorm epsilon, 1/sqrt(hd)
  // per-sequence state (b selects the row)
  int b;
  float* h;                          // [B][D]   residual stream
  float* qkv;                        // [B][(Hq+2Hkv)*hd]  raw projections
  float* attn;                       // [B][Hq*hd]
  float* z;                          // [B][F]
  float* part_o;                     // [B][Hq][S_MAX][hd]
  float* part_ml;                    // [B][Hq][S_MAX][2]
  unsigned* attn_cnt;                // [B][Hkv]  arrival counters (zero between launches)
  float2* rope_cs;                   // [B][hd/2] (cos, sin) of the current position
  int* len;                          // [B]       tokens already in the cache
  const int* page_table;             // [B][max_pages]
  const double* theta;               // [hd/2]    base^(-2d/hd)
  // embedding / head
  const void* embed;
  const void* lm_head;
  const float* g_final;
  const int* tokens;                 // [B] input token ids
  float* logits;                     // [B][V] or null
  int* token_out;                    // [B] or null
  Best* arg_part;                    // [B][ARG_MAX_WG]
  unsigned* head_cnt;                // [B]
  int advance_len;                   // 1: len[b] += 1 when the head finishes
  // layer
  const void *wq, *wk, *wv, *wo, *wg, *wu, *wd;
  const float *g_attn, *g_mlp;
  void* kv_layer;                    // this layer's page pool
  size_t page_elems;                 // elements per page = 2*Hkv*P*hd
};

constexpr int S_MAX = 64;            // upper bound on attention splits
constexpr int ARG_MAX_WG = 2048;     // upper bound on LM-head workgroups

// Position of element k of the activation vector inside LDS.  For 8-wide (bf16) weight
// vectors the two float4 halves of each group of 8 live in separate planes so that the
// 64 lanes of a wave read consecutive 16-byte words (no bank conflicts).
template <int VEC>
__device__ __forceinline__ int xs_index(int k, int K) {
  if (VEC == 8) return (((k >> 3) << 2) | (k & 3)) + ((k & 4) ? (K >> 1) : 0);
  return k;
}

// Loads x[0..K) into LDS, optionally as RMSNorm(x; gain).  red: LDS float[WAVES].
template <int VEC>
__device__ __forceinline__ void stage_x(float* xs, float* red, const float* __restrict__ x, int K,
                                        const float* __restrict__ gain, float eps) {
  float ss = 0.f;
  for (int k = threadIdx.x; k < K; k += WG) {
    const float v = x[k];
    ss = fmaf(v, v, ss);
    xs[xs_index<VEC>(k, K)] = gain ? v * gain[k] : v;
  }
  if (gain) {
    const float tot = block_sum(ss, red);
    const float r = 1.0f / sqrtf(tot / (float)K + eps);
    for (int k = threadIdx.x; k < K; k += WG) xs[xs_index<VEC>(k, K)] *= r;
  }
  __syncthreads();
}

// Dot products of R weight rows with the staged activation vector, one wave per row group.
// rowptr(r) -> pointer to row r; epi(r, sum) is called by lane 0.
template <typename WT, int R, typename RowPtr, typename Epi>
__device__ __forceinline__ void gemv_rows(int n_rows, int K, const float* xs, int gw, int tw,
                                          RowPtr rowptr, Epi epi) {
  constexpr int VEC = Vec<WT>::N;
  const int lane = threadIdx.x & 63;
  const int full = K / (64 * VEC);              // chunks in which every lane is in range
  const int ktail = full * 64 * VEC + lane * VEC;
  for (int r0 = gw * R; r0 < n_rows; r0 += tw * R) {
    const WT* rp[R];
#pragma unroll
    for (int j = 0; j < R; ++j) rp[j] = rowptr(min(r0 + j, n_rows - 1));
    float acc[R];
#pragma unroll
    for (int j = 0; j < R; ++j) acc[j] = 0.f;
#pragma unroll 2
    for (int c = 0; c < full; ++c) {
      const int k = (c * 64 + lane) * VEC;
      float wv[R][VEC];
#pragma unroll
      for (int j = 0; j < R; ++j) load_vec(rp[j] + k, wv[j]);
      float xv[VEC];
      if (VEC == 8) {
        const int q = (k >> 3) << 2;
        const float4 a = *reinterpret_cast<const float4*>(xs + q);
        const float4 b = *reinterpret_cast<const float4*>(xs + (K >> 1) + q);
        xv[0] = a.x; xv[1] = a.y; xv[2] = a.z; xv[3] = a.w;
        xv[4 % VEC] = b.x; xv[5 % VEC] = b.y; xv[6 % VEC] = b.z; xv[7 % VEC] = b.w;
      } else {
        const float4 a = *reinterpret_cast<const float4*>(xs + k);
        xv[0] = a.x; xv[1] = a.y; xv[2] = a.z; xv[3] = a.w;
      }
#pragma unroll
      for (int j = 0; j < R; ++j)
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[j] = fmaf(wv[j][e], xv[e], acc[j]);
    }
    if (ktail < K) {
      float xv[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) xv[e] = xs[xs_index<VEC>(ktail + e, K)];
#pragma unroll
      for (int j = 0; j < R; ++j) {
        float wv[VEC];
        load_vec(rp[j] + ktail, wv);
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[j] = fmaf(wv[e], xv[e], acc[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < R; ++j) acc[j] = wave_sum(acc[j]);
    if (lane == 0) {
#pragma unroll
      for (int j = 0; j < R; ++j)
        if (r0 + j < n_rows) epi(r0 + j, acc[j]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// embed: h = E[token]; (cos, sin) table of the position this token will occupy.
template <typename WT>
__device__ __forceinline__ void phase_embed(const DecParams& p) {
  const int b = p.b;
  int tok = p.tokens[b];
  tok = min(max(tok, 0), p.V - 1);
  const WT* row = reinterpret_cast<const WT*>(p.embed) + (size_t)tok * p.D;
  for (int k = threadIdx.x; k < p.D; k += WG) p.h[(size_t)b * p.D + k] = to_f32(row[k]);
  const int pos = p.len[b];
  for (int i = threadIdx.x; i < p.hd / 2; i += WG) {
    const double a = (double)pos * p.theta[i];
    p.rope_cs[(size_t)b * (p.hd / 2) + i] = make_float2((float)cos(a), (float)sin(a));
  }
}

// ---------------------------------------------------------------------------------------
// RMSNorm(h; g_attn) then the three projections, raw (un-rotated) into qkv[b].
template <typename WT>
__device__ __forceinline__ void phase_qkv(const DecParams& p, int wg, int nwg, float* smem) {
  float* xs = smem;
  float* red = smem + p.D;
  stage_x<Vec<WT>::N>(xs, red, p.h + (size_t)p.b * p.D, p.D, p.g_attn, p.eps);
  const int nq = p.Hq * p.hd, nk = p.Hkv * p.hd;
  const WT* wq = reinterpret_cast<const WT*>(p.wq);
  const WT* wk = reinterpret_cast<const WT*>(p.wk);
  const WT* wv = reinterpret_cast<const WT*>(p.wv);
  const int D = p.D;
  float* out = p.qkv + (size_t)p.b * (nq + 2 * nk);
  gemv_rows<WT, 4>(nq + 2 * nk, D, xs, wg * WAVES + (threadIdx.x >> 6), nwg * WAVES,
      [=](int r) { return r < nq ? wq + (size_t)r * D
                         : (r < nq + nk ? wk + (size_t)(r - nq) * D : wv + (size_t)(r - nq - nk) * D); },
      [=](int r, float s) { out[r] = s; });
}

// h += W x  with x read un-normalised from xin (attention output or MLP activation).
template <typename WT>
__device__ __forceinline__ void phase_proj_residual(const DecParams& p, const void* Wv, const float* xin,
                                                    int K, int wg, int nwg, float* smem) {
  float* xs = smem;
  float* red = smem + K;
  stage_x<Vec<WT>::N>(xs, red, xin, K, nullptr, 0.f);
  const WT* W = reinterpret_cast<const WT*>(Wv);
  float* h = p.h + (size_t)p.b * p.D;
  gemv_rows<WT, 4>(p.D, K, xs, wg * WAVES + (threadIdx.x >> 6), nwg * WAVES,
      [=](int r) { return W + (size_t)r * K; },
      [=](int r, float s) { h[r] += s; });
}

// z = silu(Wg y) * (Wu y),  y = RMSNorm(h; g_mlp).  Row r of both matrices in one pass.
template <typename WT>
__device__ __forceinline__ void phase_gateup(const DecParams& p, int wg, int nwg, float* smem) {
  float* xs = smem;
  float* red = smem + p.D;
  stage_x<Vec<WT>::N>(xs, red, p.h + (size_t)p.b * p.D, p.D, p.g_mlp, p.eps);
  const WT* Wg = reinterpret_cast<const WT*>(p.wg);
  const WT* Wu = reinterpret_cast<const WT*>(p.wu);
  const int D = p.D, F = p.F;
  float* z = p.z + (size_t)p.b * F;
  const int lane = threadIdx.x & 63;
  // interleave: virtual row 2r = gate row r, 2r+1 = up row r; R = 4 covers two outputs
  float keep = 0.f;
  gemv_rows<WT, 4>(2 * F, D, xs, wg * WAVES + (threadIdx.x >> 6), nwg * WAVES,
      [=](int r) { return ((r & 1) ? Wu : Wg) + (size_t)(r >> 1) * D; },
      [&](int r, float s) {
        if (r & 1) z[r >> 1] = siluf(keep) * s; else keep = s;
      });
  (void)lane;
}

// ---------------------------------------------------------------------------------------
// GQA decode attention of one (sequence, KV head, split): RoPE of q and of the new k,
// KV append, online-softmax partial over this split's keys, merge by the last arriver.
// LDS layout (floats unless noted): qs[G][hd] | knew[hd] | vnew[hd] | flag | K tile | V tile
template <typename KVT>
__device__ __forceinline__ size_t attn_smem_bytes(int G, int hd) {
  const size_t kpitch = (size_t)hd * sizeof(KVT) + 4;
  return ((size_t)G * hd + 2 * hd + 4) * sizeof(float) + 64 * kpitch + 64 * (size_t)hd * sizeof(KVT) + 16;
}

template <typename KVT>
__device__ __forceinline__ void phase_attn(const DecParams& p, int g, int s, char* smem_raw) {
  constexpr int VEC = Vec<KVT>::N;
  const int b = p.b, hd = p.hd, G = p.G, half = hd >> 1, P = p.P, S = p.S;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  float* qs = reinterpret_cast<float*>(smem_raw);
  float* knew = qs + G * hd;
  float* vnew = knew + hd;
  int* flag = reinterpret_cast<int*>(vnew + hd);
  char* kt = reinterpret_cast<char*>(flag + 4);
  const int kpitch = hd * (int)sizeof(KVT) + 4;           // bytes; odd number of 4-byte words
  KVT* vt = reinterpret_cast<KVT*>(kt + 64 * kpitch);     // 16-byte aligned: 64*kpitch % 16 == 0

  const int pos = p.len[b];
  const int nkeys = pos + 1;
  const int tiles = (nkeys + 63) >> 6;
  const int chunk = ((tiles + S - 1) / S) << 6;
  const int k_begin = s * chunk;
  const int k_end = min(nkeys, k_begin + chunk);
  const int nq = p.Hq * hd, nkv = p.Hkv * hd;
  const float* qkv = p.qkv + (size_t)b * (nq + 2 * nkv);
  const float2* cs = p.rope_cs + (size_t)b * half;
  const int* pt = p.page_table + (size_t)b * p.max_pages;
  KVT* pool = reinterpret_cast<KVT*>(p.kv_layer);
  const size_t head_off = (size_t)g * P * hd;             // within the K (or V) half of a page
  const size_t v_off = (size_t)p.Hkv * P * hd;            // V half follows the K half

  const bool active = k_begin < k_end;
  if (active) {
    // rotate q of this group's heads (pre-scaled by 1/sqrt(hd))
    for (int i = tid; i < G * half; i += WG) {
      const int hq = i / half, d = i - hq * half;
      const float x1 = qkv[(g * G + hq) * hd + d], x2 = qkv[(g * G + hq) * hd + d + half];
      const float2 c = cs[d];
      qs[hq * hd + d] = (x1 * c.x - x2 * c.y) * p.qscale;
      qs[hq * hd + d + half] = (x2 * c.x + x1 * c.y) * p.qscale;
    }
    // the split that owns the new position rotates k, rounds k and v to the cache type,
    // appends them, and keeps the stored values in LDS
    if (pos >= k_begin && pos < k_end) {
      const size_t base = (size_t)pt[pos / P] * p.page_elems + head_off + (size_t)(pos % P) * hd;
      for (int d = tid; d < half; d += WG) {
        const float x1 = qkv[nq + g * hd + d], x2 = qkv[nq + g * hd + d + half];
        const float2 c = cs[d];
        const KVT k1 = from_f32<KVT>(x1 * c.x - x2 * c.y), k2 = from_f32<KVT>(x2 * c.x + x1 * c.y);
        pool[base + d] = k1; pool[base + d + half] = k2;
        knew[d] = to_f32(k1); knew[d + half] = to_f32(k2);
      }
      for (int d = tid; d < hd; d += WG) {
        const KVT v = from_f32<KVT>(qkv[nq + nkv + g * hd + d]);
        pool[base + v_off + d] = v;
        vnew[d] = to_f32(v);
      }
    }
  }
  __syncthreads();

  constexpr int MAXH = 2;                                  // heads per wave (G <= 8)
  float m[MAXH], l[MAXH], o0[MAXH], o1[MAXH];
#pragma unroll
  for (int i = 0; i < MAXH; ++i) { m[i] = -INFINITY; l[i] = 0.f; o0[i] = 0.f; o1[i] = 0.f; }

  const int vec_per_key = hd / VEC;
  for (int t0 = k_begin; t0 < k_end; t0 += 64) {
    // stage 64 keys of K (padded rows) and V
    for (int i = tid; i < 64 * vec_per_key; i += WG) {
      const int j = i / vec_per_key, c = (i - j * vec_per_key) * VEC;
      const int key = t0 + j;
      uint4 kv4 = make_uint4(0, 0, 0, 0), vv4 = make_uint4(0, 0, 0, 0);
      bool fresh = false;
      if (key < k_end) {
        if (key == pos) fresh = true;
        else {
          const size_t base = (size_t)pt[key / P] * p.page_elems + head_off + (size_t)(key % P) * hd + c;
          kv4 = *reinterpret_cast<const uint4*>(pool + base);
          vv4 = *reinterpret_cast<const uint4*>(pool + base + v_off);
        }
      }
      if (fresh) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          *reinterpret_cast<KVT*>(kt + j * kpitch + (c + e) * sizeof(KVT)) = from_f32<KVT>(knew[c + e]);
          vt[j * hd + c + e] = from_f32<KVT>(vnew[c + e]);
        }
      } else {
        uint32_t* kd = reinterpret_cast<uint32_t*>(kt + j * kpitch + c * sizeof(KVT));
        kd[0] = kv4.x; kd[1] = kv4.y; kd[2] = kv4.z; kd[3] = kv4.w;
        *reinterpret_cast<uint4*>(vt + j * hd + c) = vv4;
      }
    }
    __syncthreads();
    const int jn = min(64, k_end - t0);
#pragma unroll
    for (int hi = 0; hi < MAXH; ++hi) {
      const int hq = wave + hi * WAVES;
      if (hq < G) {
        // score of key t0+lane against head hq
        float sc = 0.f;
        const char* krow = kt + lane * kpitch;
        const float* q = qs + hq * hd;
        if (sizeof(KVT) == 2) {
          for (int d = 0; d < hd; d += 2) {
            const uint32_t w2 = *reinterpret_cast<const uint32_t*>(krow + d * 2);
            sc = fmaf(q[d], __uint_as_float(w2 << 16), sc);
            sc = fmaf(q[d + 1], __uint_as_float(w2 & 0xffff0000u), sc);
          }
        } else {
          for (int d = 0; d < hd; ++d) sc = fmaf(q[d], *reinterpret_cast<const float*>(krow + d * 4), sc);
        }
        if (lane >= jn) sc = -INFINITY;
        const float mt = wave_max(sc);
        const float mn = fmaxf(m[hi], mt);
        const float corr = expf(m[hi] - mn);               // exp(-inf) = 0 on the first tile
        const float pj = (lane < jn) ? expf(sc - mn) : 0.f;
        l[hi] = l[hi] * corr + wave_sum(pj);
        o0[hi] *= corr; o1[hi] *= corr;
        m[hi] = mn;
        // o += p_j * V[j]; lane owns dims lane and lane+64
        for (int j = 0; j < jn; ++j) {
          const float pb = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pj), j));
          if (lane < hd) o0[hi] = fmaf(pb, to_f32(vt[j * hd + lane]), o0[hi]);
          if (lane + 64 < hd) o1[hi] = fmaf(pb, to_f32(vt[j * hd + lane + 64]), o1[hi]);
        }
      }
    }
    __syncthreads();
  }

  // partial results of this split
#pragma unroll
  for (int hi = 0; hi < MAXH; ++hi) {
    const int hq = wave + hi * WAVES;
    if (hq < G) {
      const int H = g * G + hq;
      float* po = p.part_o + (((size_t)b * p.Hq + H) * S_MAX + s) * hd;
      if (lane < hd) po[lane] = o0[hi];
      if (lane + 64 < hd) po[lane + 64] = o1[hi];
      if (lane == 0) {
        float* pml = p.part_ml + (((size_t)b * p.Hq + H) * S_MAX + s) * 2;
        pml[0] = m[hi]; pml[1] = l[hi];
      }
    }
  }
  // the last split to arrive merges all of them in split order (result independent of
  // arrival order)
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const unsigned old = atomicAdd(&p.attn_cnt[b * p.Hkv + g], 1u);
    const int last = (old == (unsigned)(S - 1));
    if (last) p.attn_cnt[b * p.Hkv + g] = 0u;
    *flag = last;
  }
  __syncthreads();
  if (*flag) {
    __threadfence();
#pragma unroll
    for (int hi = 0; hi < MAXH; ++hi) {
      const int hq = wave + hi * WAVES;
      if (hq < G) {
        const int H = g * G + hq;
        const float* pml = p.part_ml + ((size_t)b * p.Hq + H) * S_MAX * 2;
        const float* po = p.part_o + ((size_t)b * p.Hq + H) * S_MAX * hd;
        float M = -INFINITY;
        for (int t = 0; t < S; ++t) M = fmaxf(M, __builtin_nontemporal_load(pml + 2 * t));
        float den = 0.f, a0 = 0.f, a1 = 0.f;
        for (int t = 0; t < S; ++t) {
          const float mt = __builtin_nontemporal_load(pml + 2 * t);
          const float lt = __builtin_nontemporal_load(pml + 2 * t + 1);
          if (lt > 0.f) {
            const float w = expf(mt - M);
            den = fmaf(lt, w, den);
            if (lane < hd) a0 = fmaf(__builtin_nontemporal_load(po + t * hd + lane), w, a0);
            if (lane + 64 < hd) a1 = fmaf(__builtin_nontemporal_load(po + t * hd + lane + 64), w, a1);
          }
        }
        float* out = p.attn + (size_t)b * nq + H * hd;
        if (lane < hd) out[lane] = a0 / den;
        if (lane + 64 < hd) out[lane + 64] = a1 / den;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// logits = W_lm RMSNorm(h; g_final); greedy token by a two-level argmax whose last arriver
// also advances the sequence length.
template <typename WT>
__device__ __forceinline__ void phase_head(const DecParams& p, int wg, int nwg, float* smem) {
  float* xs = smem;
  float* red = smem + p.D;
  Best* wbest = reinterpret_cast<Best*>(red + WAVES);
  int* flag = reinterpret_cast<int*>(wbest + WAVES);
  const int b = p.b, D = p.D, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  stage_x<Vec<WT>::N>(xs, red, p.h + (size_t)b * D, D, p.g_final, p.eps);
  const WT* W = reinterpret_cast<const WT*>(p.lm_head);
  float* lg = p.logits ? p.logits + (size_t)b * p.V : nullptr;
  Best best{-INFINITY, 0x7fffffff};
  gemv_rows<WT, 4>(p.V, D, xs, wg * WAVES + wave, nwg * WAVES,
      [=](int r) { return W + (size_t)r * D; },
      [&](int r, float s) {
        if (lg) lg[r] = s;
        const Best c{s, r};
        if (better(c, best)) best = c;
      });
  if (lane == 0) wbest[wave] = best;
  __syncthreads();
  if (tid == 0) {
    Best bb = wbest[0];
    for (int w = 1; w < WAVES; ++w) if (better(wbest[w], bb)) bb = wbest[w];
    p.arg_part[(size_t)b * ARG_MAX_WG + wg] = bb;
    __threadfence();
    const unsigned old = atomicAdd(&p.head_cnt[b], 1u);
    const int last = (old == (unsigned)(nwg - 1));
    if (last) p.head_cnt[b] = 0u;
    *flag = last;
  }
  __syncthreads();
  if (*flag) {
    __threadfence();
    Best bb{-INFINITY, 0x7fffffff};
    const float* ap = reinterpret_cast<const float*>(p.arg_part + (size_t)b * ARG_MAX_WG);
    const int* api = reinterpret_cast<const int*>(ap);
    for (int i = tid; i < nwg; i += WG) {
      const Best c{__builtin_nontemporal_load(ap + 2 * i), __builtin_nontemporal_load(api + 2 * i + 1)};
      if (better(c, bb)) bb = c;
    }
    // butterfly over the wave, then over the waves
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const Best c{__shfl_xor(bb.v, o, 64), __shfl_xor(bb.i, o, 64)};
      if (better(c, bb)) bb = c;
    }
    __syncthreads();
    if (lane == 0) wbest[wave] = bb;
    __syncthreads();
    if (tid == 0) {
      Best r = wbest[0];
      for (int w = 1; w < WAVES; ++w) if (better(wbest[w], r)) r = wbest[w];
      if (p.token_out) p.token_out[b] = r.i;
      if (p.advance_len) p.len[b] += 1;
    }
  }
}

// ---------------------------------------------------------------------------------------
// one kernel per fused op
template <typename WT> __global__ void __launch_bounds__(WG) k_embed(DecParams p) { phase_embed<WT>(p); }

template <typename WT> __global__ void __launch_bounds__(WG) k_qkv(DecParams p) {
  extern __shared__ __align__(16) float smem_f[];
  phase_qkv<WT>(p, blockIdx.x, gridDim.x, smem_f);
}
template <typename WT> __global__ void __launch_bounds__(WG) k_attn(DecParams p) {
  extern __shared__ __align__(16) float smem_f[];
  phase_attn<WT>(p, blockIdx.y, blockIdx.x, reinterpret_cast<char*>(smem_f));
}
template <typename WT> __global__ void __launch_bounds__(WG) k_oproj(DecParams p) {
  extern __shared__ __align__(16) float smem_f[];
  phase_proj_residual<WT>(p, p.wo, p.attn + (size_t)p.b * p.Hq * p.hd, p.Hq * p.hd, blockIdx.x, gridDim.x, smem_f);
}
template <typename WT> __global__ void __launch_bounds__(WG) k_gateup(DecParams p) {
  extern __shared__ __align__(16) float smem_f[];
  phase_gateup<WT>(p, blockIdx.x, gridDim.x, smem_f);
}
template <typename WT> __global__ void __launch_bounds__(WG) k_down(DecParams p) {
  extern __shared__ __align__(16) float smem_f[];
  phase_proj_residual<WT>(p, p.wd, p.z + (size_t)p.b * p.F, p.F, blockIdx.x, gridDim.x, smem_f);
}
template <typename WT> __global__ void __launch_bounds__(WG) k_head(DecParams p) {
  extern __shared__ __align__(16) float smem_f[];
  phase_head<WT>(p, blockIdx.x, gridDim.x, smem_f);
}

// Stand-alone mat-vec (unit tests and kernel-level roofline): y (+)= W x.
template <typename WT> __global__ void __launch_bounds__(WG)
k_gemv(const WT* __restrict__ W, const float* __restrict__ x, float* __restrict__ y, int n, int K, int accumulate) {
  extern __shared__ __align__(16) float smem_f[];
  stage_x<Vec<WT>::N>(smem_f, smem_f + K, x, K, nullptr, 0.f);
  gemv_rows<WT, 4>(n, K, smem_f, blockIdx.x * WAVES + (threadIdx.x >> 6), gridDim.x * WAVES,
      [=](int r) { return W + (size_t)r * K; },
      [=](int r, float s) { y[r] = accumulate ? y[r] + s : s; });
}

}  // namespace first
