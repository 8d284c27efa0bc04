// Whole decode step of one sequence as ONE persistent kernel (bf16 models, batch 1):
// one 512-thread workgroup per compute unit (256 VGPRs per lane for deep prefetch), phases separated by grid-wide barriers, and
// the weights of the next phase requested from HBM before each barrier so the memory system
// never drains while workgroups wait.  Kept-layer indices are read from the device-side
// compaction, so a skipped layer costs neither a launch nor a byte (Section 4.3 item 2).
#pragma once
#include "decode_kernels.h"

namespace first {

constexpr int SK_THREADS = 512;
constexpr int SK_WAVES = SK_THREADS / 64;
constexpr int SK_SEG = 2048;          // elements of a weight row handled by one wave at a time (4 x 16 B per lane)
constexpr int SK_PD = 8;              // row segments in flight per wave (32 KB)
constexpr int SK_PD_ATT = 4;          // ring slots kept in flight across the attention phase
constexpr int SK_PSUM = 2048;         // partial sums a workgroup can hold (row segments per phase)
constexpr int SK_SMAX = 8;            // attention splits merged by the O-projection prologue
constexpr unsigned SK_SPIN_LIMIT = 1u << 21;

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// Pointers that come out of a struct in memory are "generic" to the compiler and would be
// read with flat instructions (which also tick the LDS wait counter); these helpers state
// that the address is global memory.
#define SK_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ const SK_GLOBAL T* as_global(const T* p) {
  return reinterpret_cast<const SK_GLOBAL T*>(reinterpret_cast<unsigned long long>(p));
}
template <typename T>
__device__ __forceinline__ SK_GLOBAL T* as_global(T* p) {
  return reinterpret_cast<SK_GLOBAL T*>(reinterpret_cast<unsigned long long>(p));
}
// 16-byte streaming load (weights are read once per step: do not keep them in cache).
__device__ __forceinline__ uint4 ld_stream16(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4_t*>(p)));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 ld_global16(const void* p) {
  const u32x4_t v = *as_global(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float ldg(const float* p) { return *as_global(p); }
__device__ __forceinline__ void stg_bf16(bf16* p, bf16 v) { *as_global(&p->v) = v.v; }

struct LayerDev {
  const bf16 *wq, *wk, *wv, *wo, *wg, *wu, *wd;
  const float *g_attn, *g_mlp;
  bf16* kv;
};

// Values loaded from global memory that are the same for every lane: tell the compiler so
// (keeps them in scalar registers instead of one copy per lane).
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T>
__device__ __forceinline__ T* uni(T* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<T*>(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ LayerDev load_layer(const LayerDev* arr, int i) {
  LayerDev l = arr[i];
  l.wq = uni(l.wq); l.wk = uni(l.wk); l.wv = uni(l.wv); l.wo = uni(l.wo); l.wg = uni(l.wg); l.wu = uni(l.wu);
  l.wd = uni(l.wd); l.g_attn = uni(l.g_attn); l.g_mlp = uni(l.g_mlp); l.kv = uni(l.kv);
  return l;
}

struct StepParams {
  DecParams d;                 // geometry, workspaces, sequence slot (layer fields unused)
  const LayerDev* layers;      // [L]
  const int* kept;             // [B][L] ascending kept-layer indices
  const int* n_kept;           // [B]
  int L;
  unsigned* bar;               // grid barrier counter, zero at launch
  int* err;                    // set to 1 if a barrier wait gives up
};

// LDS carve-up (floats)
struct SkLds {
  float* xs;      // [max(D, Hq*hd)] activation vector of the running phase
  float* zs;      // [F] MLP activation for the down projection
  float* psum;    // [SK_PSUM]
  float* red;     // [SK_WAVES + 8]
  float* qs;      // [G*hd] rotated, pre-scaled queries of this workgroup's KV head
  float* knew;    // [hd]
  float* vnew;    // [hd]
  float2* cs;     // [hd/2]
  float* ps;      // [SK_WAVES][64]
  float* mb;      // [SK_WAVES][hd + 2]
  int* flag;      // [4]
};

__host__ __device__ inline size_t sk_lds_floats(int D, int nq, int F, int G, int hd) {
  const int xs = D > nq ? D : nq;
  return (size_t)xs + F + SK_PSUM + (SK_WAVES + 8) + (size_t)G * hd + 2 * hd + hd + SK_WAVES * 64 +
         (size_t)SK_WAVES * (hd + 2) + 4;
}

__device__ __forceinline__ SkLds sk_carve(float* base, int D, int nq, int F, int G, int hd) {
  SkLds s;
  const int xs = D > nq ? D : nq;
  s.xs = base; base += xs;
  s.zs = base; base += F;
  s.psum = base; base += SK_PSUM;
  s.red = base; base += SK_WAVES + 8;
  s.qs = base; base += G * hd;
  s.knew = base; base += hd;
  s.vnew = base; base += hd;
  s.cs = reinterpret_cast<float2*>(base); base += hd;
  s.ps = base; base += SK_WAVES * 64;
  s.mb = base; base += SK_WAVES * (hd + 2);
  s.flag = reinterpret_cast<int*>(base);
  return s;
}

// Arrive-and-wait over all workgroups.  Every thread releases its writes, thread 0 arrives
// and polls with a bounded spin; a wait that gives up (or sees another workgroup's give-up
// flag) makes the whole workgroup return false so that every wave still exits.
__device__ __forceinline__ bool grid_barrier(unsigned* bar, int* err, unsigned target, int* flag) {
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(bar, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned spins = 0;
    int good = 1;
    while (__hip_atomic_load(bar, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      __builtin_amdgcn_s_sleep(1);
      if (++spins > SK_SPIN_LIMIT || __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
        __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        good = 0;
        break;
      }
    }
    *flag = good;
  }
  __syncthreads();
  __threadfence();
  return *flag != 0;
}

// Sum over the workgroup's threads in a fixed order; every thread gets the total.
__device__ __forceinline__ float sk_block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < SK_WAVES; ++w) t += red[w];
  return t;
}

// xs <- x or RMSNorm(x; gain), in the two-plane layout the 8-wide weight vectors read.
__device__ __forceinline__ void sk_stage(float* xs, float* red, const float* x, int K, const float* gain, float eps) {
  float ss = 0.f;
  for (int k = threadIdx.x; k < K; k += SK_THREADS) {
    const float v = ldg(x + k);
    ss = fmaf(v, v, ss);
    xs[xs_index<8>(k, K)] = gain ? v * ldg(gain + k) : v;
  }
  if (gain) {
    const float tot = sk_block_sum(ss, red);
    const float r = 1.0f / sqrtf(tot / (float)K + eps);
    for (int k = threadIdx.x; k < K; k += SK_THREADS) xs[xs_index<8>(k, K)] *= r;
  }
  __syncthreads();
}

// A segment is one mat-vec phase of the step (QKV, O, gate/up, down of a kept layer, or the
// LM head).  Rows [row0, row0+nrows) of its [N, K] matrix belong to this workgroup; a unit
// is one 2048-element piece of one row and goes to wave (unit % SK_WAVES) in round
// (unit / SK_WAVES).  The number of rounds is padded to a multiple of SK_PD so that the ring
// of in-flight loads keeps a static register assignment across segments.
enum { SEG_QKV = 0, SEG_O = 1, SEG_GU = 2, SEG_DN = 3, SEG_HEAD = 4, SEG_NONE = 5 };
struct SegDesc {
  const bf16 *m0, *m1, *m2;     // up to three stacked matrices (or two interleaved ones)
  int n0, n1, K, inter;
  int row0, nrows, nseg, nunits, nr_pad;
  int kind;
  const float* gain;            // RMSNorm gain of the phase's input (null: no norm)
  bf16* kv;                     // KV pool of the layer (attention precedes SEG_O)
};

__device__ __forceinline__ void seg_split(SegDesc& d, int N, int K, int cu, int ncu, int pair) {
  const int n = N / pair;
  d.K = K;
  d.row0 = (int)(((long long)n * cu) / ncu) * pair;
  d.nrows = (int)(((long long)n * (cu + 1)) / ncu) * pair - d.row0;
  d.nseg = K / SK_SEG;
  d.nunits = d.nrows * d.nseg;
  const int nr = (d.nunits + SK_WAVES - 1) / SK_WAVES;
  d.nr_pad = max(SK_PD, (nr + SK_PD - 1) / SK_PD * SK_PD);
}

__device__ __forceinline__ SegDesc seg_desc(const StepParams& P, int s, int nk, const int* kept, int cu, int ncu) {
  const DecParams& p = P.d;
  const int nq = p.Hq * p.hd, nkv = p.Hkv * p.hd;
  SegDesc d{};
  d.kind = SEG_NONE;
  if (s > 4 * nk) return d;
  if (s == 4 * nk) {
    d.kind = SEG_HEAD; d.m0 = reinterpret_cast<const bf16*>(p.lm_head); d.n0 = p.V; d.gain = p.g_final;
    seg_split(d, p.V, p.D, cu, ncu, 1);
    return d;
  }
  const LayerDev lw = load_layer(P.layers, uni(kept[s >> 2]));
  d.kind = s & 3;
  d.kv = lw.kv;
  switch (d.kind) {
    case SEG_QKV:
      d.m0 = lw.wq; d.m1 = lw.wk; d.m2 = lw.wv; d.n0 = nq; d.n1 = nkv; d.gain = lw.g_attn;
      seg_split(d, nq + 2 * nkv, p.D, cu, ncu, 1);
      break;
    case SEG_O:
      d.m0 = lw.wo; d.n0 = p.D;
      seg_split(d, p.D, nq, cu, ncu, 1);
      break;
    case SEG_GU:
      d.m0 = lw.wg; d.m1 = lw.wu; d.inter = 1; d.gain = lw.g_mlp;
      seg_split(d, 2 * p.F, p.D, cu, ncu, 2);
      break;
    default:
      d.m0 = lw.wd; d.n0 = p.D;
      seg_split(d, p.D, p.F, cu, ncu, 1);
      break;
  }
  return d;
}

__device__ __forceinline__ const bf16* seg_row(const SegDesc& d, int r) {
  if (d.inter) return ((r & 1) ? d.m1 : d.m0) + (size_t)(r >> 1) * d.K;
  if (r < d.n0) return d.m0 + (size_t)r * d.K;
  if (r < d.n0 + d.n1) return d.m1 + (size_t)(r - d.n0) * d.K;
  return d.m2 + (size_t)(r - d.n0 - d.n1) * d.K;
}

// Requests one round (4 x 16 B per lane) of a segment into a ring slot.
__device__ __forceinline__ void sk_issue(const SegDesc& d, int round, uint4 (&b)[4]) {
  const int u = round * SK_WAVES + (threadIdx.x >> 6);
  if (d.kind != SEG_NONE && u < d.nunits) {
    const int rl = u / d.nseg, sg = u - rl * d.nseg;
    const bf16* p = seg_row(d, d.row0 + rl) + (size_t)sg * SK_SEG + (threadIdx.x & 63) * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = ld_stream16(p + j * 512);
  }
}

// Dot product of one ring slot with the staged activation vector -> psum[unit].
__device__ __forceinline__ void sk_consume(const SegDesc& d, int round, const uint4 (&b)[4], const float* xs,
                                           float* psum) {
  const int u = round * SK_WAVES + (threadIdx.x >> 6);
  if (u < d.nunits) {
    const int lane = threadIdx.x & 63, K = d.K;
    const int rl = u / d.nseg, sg = u - rl * d.nseg;
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = sg * SK_SEG + j * 512 + lane * 8;
      const int q = (k >> 3) << 2;
      const float4 x0 = *reinterpret_cast<const float4*>(xs + q);
      const float4 x1 = *reinterpret_cast<const float4*>(xs + (K >> 1) + q);
      const uint4 w = b[j];
      acc = fmaf(__uint_as_float(w.x << 16), x0.x, acc); acc = fmaf(__uint_as_float(w.x & 0xffff0000u), x0.y, acc);
      acc = fmaf(__uint_as_float(w.y << 16), x0.z, acc); acc = fmaf(__uint_as_float(w.y & 0xffff0000u), x0.w, acc);
      acc = fmaf(__uint_as_float(w.z << 16), x1.x, acc); acc = fmaf(__uint_as_float(w.z & 0xffff0000u), x1.y, acc);
      acc = fmaf(__uint_as_float(w.w << 16), x1.z, acc); acc = fmaf(__uint_as_float(w.w & 0xffff0000u), x1.w, acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) psum[u] = acc;
  }
}

__device__ __forceinline__ float sk_row_sum(const float* psum, int rl, int nseg) {
  float s = 0.f;
  for (int g = 0; g < nseg; ++g) s += psum[rl * nseg + g];
  return s;
}

// ---------------------------------------------------------------------------------------
// Attention of workgroup (KV head g, split s): the waves = G query heads x (SK_WAVES/G) key groups,
// lane = key for the scores, lane = (key subgroup, 8-dim chunk) for the weighted values.
template <int HD>
__device__ __forceinline__ void sk_attention(const StepParams& P, bf16* pool, const SkLds& S, int g, int s, int nsplit) {
  const DecParams& p = P.d;
  constexpr int HALF = HD / 2, LPR = HD / 8, RPI = 64 / LPR;   // lanes per V row, V rows per load
  const int b = p.b, G = p.G, Pg = p.P;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hq = wave % G, kg = wave / G, nkg = SK_WAVES / G;
  const int pos = uni(p.len[b]), nkeys = pos + 1, tiles = (nkeys + 63) >> 6;
  const int tps = (tiles + nsplit - 1) / nsplit;
  const int t_first = s * tps, t_last = min(tiles, t_first + tps);
  const int nq = p.Hq * HD, nkv = p.Hkv * HD;
  const float* qkv = p.qkv + (size_t)b * (nq + 2 * nkv);
  const int* pt = p.page_table + (size_t)b * p.max_pages;
  const size_t head_off = (size_t)g * Pg * HD, v_off = (size_t)p.Hkv * Pg * HD;
  const bool owns_new = (pos >> 6) >= t_first && (pos >> 6) < t_last;

  // rotated queries of the G heads (pre-scaled), and the new key / value as stored
  for (int i = tid; i < G * HALF; i += SK_THREADS) {
    const int h = i / HALF, d = i - h * HALF;
    const float x1 = qkv[(g * G + h) * HD + d], x2 = qkv[(g * G + h) * HD + d + HALF];
    const float2 c = S.cs[d];
    S.qs[h * HD + d] = (x1 * c.x - x2 * c.y) * p.qscale;
    S.qs[h * HD + d + HALF] = (x2 * c.x + x1 * c.y) * p.qscale;
  }
  if (owns_new) {
    const size_t base = (size_t)pt[pos / Pg] * p.page_elems + head_off + (size_t)(pos % Pg) * HD;
    for (int d = tid; d < HALF; d += SK_THREADS) {
      const float x1 = qkv[nq + g * HD + d], x2 = qkv[nq + g * HD + d + HALF];
      const float2 c = S.cs[d];
      const bf16 k1 = from_f32<bf16>(x1 * c.x - x2 * c.y), k2 = from_f32<bf16>(x2 * c.x + x1 * c.y);
      stg_bf16(pool + base + d, k1); stg_bf16(pool + base + d + HALF, k2);
      S.knew[d] = to_f32(k1); S.knew[d + HALF] = to_f32(k2);
    }
    for (int d = tid; d < HD; d += SK_THREADS) {
      const bf16 v = from_f32<bf16>(qkv[nq + nkv + g * HD + d]);
      stg_bf16(pool + base + v_off + d, v);
      S.vnew[d] = to_f32(v);
    }
  }
  __syncthreads();

  float m = -INFINITY, l = 0.f, o[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = 0.f;
  const float* q = S.qs + hq * HD;
  float* ps = S.ps + wave * 64;
  const int sub = lane / LPR, dc = lane % LPR;

  for (int t = t_first + kg; t < t_last; t += nkg) {
    const int t0 = t << 6;
    const int key = t0 + lane;
    const bool valid = key < nkeys;
    const int ksafe = valid ? key : pos;
    const bf16* krow = pool + (size_t)pt[ksafe / Pg] * p.page_elems + head_off + (size_t)(ksafe % Pg) * HD;
    float sc = 0.f;
#pragma unroll
    for (int hf = 0; hf < HD / 32; ++hf) {             // 32 dims (4 x 16 B) of the key row at a time
      uint4 kr[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) kr[c] = ld_global16(krow + hf * 32 + c * 8);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float4 q0 = *reinterpret_cast<const float4*>(q + hf * 32 + c * 8);
        const float4 q1 = *reinterpret_cast<const float4*>(q + hf * 32 + c * 8 + 4);
        const uint4 w = kr[c];
        sc = fmaf(__uint_as_float(w.x << 16), q0.x, sc); sc = fmaf(__uint_as_float(w.x & 0xffff0000u), q0.y, sc);
        sc = fmaf(__uint_as_float(w.y << 16), q0.z, sc); sc = fmaf(__uint_as_float(w.y & 0xffff0000u), q0.w, sc);
        sc = fmaf(__uint_as_float(w.z << 16), q1.x, sc); sc = fmaf(__uint_as_float(w.z & 0xffff0000u), q1.y, sc);
        sc = fmaf(__uint_as_float(w.w << 16), q1.z, sc); sc = fmaf(__uint_as_float(w.w & 0xffff0000u), q1.w, sc);
      }
    }
    if (t0 <= pos && pos < t0 + 64) {
      // the key appended in this step: take it from LDS (the stored, rounded value)
      float part = 0.f;
      for (int d = lane; d < HD; d += 64) part = fmaf(q[d], S.knew[d], part);
      part = wave_sum(part);
      if (key == pos) sc = part;
    }
    if (!valid) sc = -INFINITY;
    const float mn = fmaxf(m, wave_max(sc));
    const float corr = expf(m - mn);
    const float pj = valid ? expf(sc - mn) : 0.f;
    l = l * corr + wave_sum(pj);
    m = mn;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] *= corr;
    ps[lane] = pj;
    // weighted values: load i covers keys t0 + RPI*i + sub, dims dc*8 .. dc*8+7
#pragma unroll
    for (int vh = 0; vh < LPR / 4; ++vh) {
      uint4 vr[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kv = t0 + RPI * (vh * 4 + i) + sub;
        const int kvs = kv < nkeys ? kv : pos;
        vr[i] = ld_global16(pool + (size_t)pt[kvs / Pg] * p.page_elems + head_off + v_off + (size_t)(kvs % Pg) * HD +
                            dc * 8);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int jj = RPI * (vh * 4 + i) + sub;
        const float pw = ps[jj];
        float v[8];
        const uint4 w = vr[i];
        v[0] = __uint_as_float(w.x << 16); v[1] = __uint_as_float(w.x & 0xffff0000u);
        v[2] = __uint_as_float(w.y << 16); v[3] = __uint_as_float(w.y & 0xffff0000u);
        v[4] = __uint_as_float(w.z << 16); v[5] = __uint_as_float(w.z & 0xffff0000u);
        v[6] = __uint_as_float(w.w << 16); v[7] = __uint_as_float(w.w & 0xffff0000u);
        if (t0 + jj == pos) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = S.vnew[dc * 8 + e];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = fmaf(pw, v[e], o[e]);
      }
    }
  }
  // fold the key subgroups: afterwards lanes 0..LPR-1 hold dims lane*8 .. lane*8+7
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] += __shfl_xor(o[e], off, 64);
  float* mb = S.mb + wave * (HD + 2);
  if (lane < LPR) {
#pragma unroll
    for (int e = 0; e < 8; ++e) mb[lane * 8 + e] = o[e];
  }
  if (lane == 0) { mb[HD] = m; mb[HD + 1] = l; }
  __syncthreads();
  // key group 0 of each head merges the groups in order and writes the split's partial
  if (kg == 0) {
    float M = -INFINITY;
    for (int k2 = 0; k2 < nkg; ++k2) M = fmaxf(M, S.mb[(k2 * G + hq) * (HD + 2) + HD]);
    float den = 0.f, a0 = 0.f, a1 = 0.f;
    for (int k2 = 0; k2 < nkg; ++k2) {
      const float* src = S.mb + (k2 * G + hq) * (HD + 2);
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
    po[lane] = a0;
    if (HD > 64) po[lane + 64] = a1;
    if (lane == 0) {
      float* pml = p.part_ml + (((size_t)b * p.Hq + H) * S_MAX + s) * 2;
      pml[0] = M; pml[1] = den;
    }
  }
}

// xs <- attention output merged over the splits (fixed order), two-plane layout.
__device__ __forceinline__ void sk_stage_attn(const StepParams& P, const SkLds& S, int nsplit) {
  const DecParams& p = P.d;
  const int nq = p.Hq * p.hd;
  for (int e = threadIdx.x; e < nq; e += SK_THREADS) {
    const int H = e / p.hd, d = e - H * p.hd;
    const float* pml = p.part_ml + ((size_t)p.b * p.Hq + H) * S_MAX * 2;
    const float* po = p.part_o + ((size_t)p.b * p.Hq + H) * S_MAX * p.hd;
    float M = -INFINITY;
    for (int t = 0; t < nsplit; ++t) M = fmaxf(M, pml[2 * t]);
    float den = 0.f, a = 0.f;
    for (int t = 0; t < nsplit; ++t) {
      const float lt = pml[2 * t + 1];
      if (lt > 0.f) {
        const float w = expf(pml[2 * t] - M);
        den = fmaf(lt, w, den);
        a = fmaf(po[t * p.hd + d], w, a);
      }
    }
    S.xs[xs_index<8>(e, nq)] = a / den;
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------------------
template <int HD>
__global__ void __launch_bounds__(SK_THREADS) k_step(StepParams P) {
  extern __shared__ __align__(16) float smem_f[];
  const DecParams& p = P.d;
  const int cu = blockIdx.x, ncu = gridDim.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int b = p.b, D = p.D, F = p.F, nq = p.Hq * HD, nkv = p.Hkv * HD;
  const SkLds S = sk_carve(smem_f, D, nq, F, p.G, HD);
  uint4 buf[SK_PD][4];
  unsigned bar_target = 0;
  float* h = p.h + (size_t)b * D;
  const int nk = uni(P.n_kept[b]);
  const int* kept = P.kept + (size_t)b * P.L;
  const int pos = uni(p.len[b]);
  const int nkeys = pos + 1, tiles = (nkeys + 63) >> 6;
  // attention splits: enough workgroups that each wave sees about one 64-key tile
  const int nkg = SK_WAVES / p.G;
  int nsplit = (tiles + nkg - 1) / nkg;
  nsplit = max(1, min(nsplit, min(SK_SMAX, ncu / p.Hkv)));

#define SK_BARRIER()                                                                   \
  do {                                                                                 \
    bar_target += (unsigned)ncu;                                                       \
    if (!grid_barrier(P.bar, P.err, bar_target, S.flag)) return;                       \
  } while (0)

  // ---- h = E[token]; rotation table of this position (kept in LDS for the whole step)
  {
    int tok = uni(p.tokens[b]);
    tok = min(max(tok, 0), p.V - 1);
    const bf16* row = reinterpret_cast<const bf16*>(p.embed) + (size_t)tok * D;
    const int r0 = (int)(((long long)D * cu) / ncu), r1 = (int)(((long long)D * (cu + 1)) / ncu);
    for (int k = r0 + tid; k < r1; k += SK_THREADS) h[k] = to_f32(row[k]);
    for (int i = tid; i < HD / 2; i += SK_THREADS) {
      const double a = (double)pos * p.theta[i];
      S.cs[i] = make_float2((float)cos(a), (float)sin(a));
    }
  }

  // ---- the segments: one ring of SK_PD in-flight rounds per wave runs through all of them
  const int nsegs = 4 * nk + 1;
  SegDesc cur = seg_desc(P, 0, nk, kept, cu, ncu);
  SegDesc nxt = seg_desc(P, 1, nk, kept, cu, ncu);
#pragma unroll
  for (int j = 0; j < SK_PD; ++j) sk_issue(cur, j, buf[j]);

  for (int s = 0; s < nsegs; ++s) {
    // -- entering the segment: everything it reads was written before this barrier
    SK_BARRIER();
    const float* xsrc = S.xs;
    if (cur.kind == SEG_O) {
      // only SK_PD_ATT ring slots stay in flight across attention (it needs the registers);
      // the upper slots hold nothing here and are refilled right after
#pragma unroll
      for (int j = SK_PD_ATT; j < SK_PD; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) buf[j][i] = make_uint4(0, 0, 0, 0);
      if (cu < p.Hkv * nsplit) sk_attention<HD>(P, cur.kv, S, cu / nsplit, cu % nsplit, nsplit);
#pragma unroll
      for (int j = SK_PD_ATT; j < SK_PD; ++j) sk_issue(cur, j, buf[j]);
      SK_BARRIER();
      sk_stage_attn(P, S, nsplit);
    } else if (cur.kind == SEG_DN) {
      sk_stage(S.zs, S.red, p.z + (size_t)b * F, F, nullptr, 0.f);
      xsrc = S.zs;
    } else {
      sk_stage(S.xs, S.red, h, D, cur.gain, p.eps);
    }
    // -- stream the segment's weights through the ring
    for (int r0 = 0; r0 < cur.nr_pad; r0 += SK_PD) {
#pragma unroll
      for (int j = 0; j < SK_PD; ++j) {
        sk_consume(cur, r0 + j, buf[j], xsrc, S.psum);
        const int t = r0 + j + SK_PD;
        if (t < cur.nr_pad) sk_issue(cur, t, buf[j]);
        else if (nxt.kind != SEG_O || j < SK_PD_ATT) sk_issue(nxt, t - cur.nr_pad, buf[j]);
      }
    }
    __syncthreads();
    // -- results of the segment
    if (cur.kind == SEG_QKV) {
      float* out = p.qkv + (size_t)b * (nq + 2 * nkv);
      for (int r = tid; r < cur.nrows; r += SK_THREADS) out[cur.row0 + r] = sk_row_sum(S.psum, r, cur.nseg);
    } else if (cur.kind == SEG_O || cur.kind == SEG_DN) {
      for (int r = tid; r < cur.nrows; r += SK_THREADS) h[cur.row0 + r] += sk_row_sum(S.psum, r, cur.nseg);
    } else if (cur.kind == SEG_GU) {
      float* z = p.z + (size_t)b * F;
      for (int r = tid; r < cur.nrows / 2; r += SK_THREADS) {
        const float gt = sk_row_sum(S.psum, 2 * r, cur.nseg), up = sk_row_sum(S.psum, 2 * r + 1, cur.nseg);
        z[cur.row0 / 2 + r] = siluf(gt) * up;
      }
    } else {
      float* lg = p.logits ? p.logits + (size_t)b * p.V : nullptr;
      Best best{-INFINITY, 0x7fffffff};
      for (int r = tid; r < cur.nrows; r += SK_THREADS) {
        const float v = sk_row_sum(S.psum, r, cur.nseg);
        if (lg) lg[cur.row0 + r] = v;
        const Best c{v, cur.row0 + r};
        if (better(c, best)) best = c;
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const Best c{__shfl_xor(best.v, o, 64), __shfl_xor(best.i, o, 64)};
        if (better(c, best)) best = c;
      }
      Best* wb = reinterpret_cast<Best*>(S.psum);          // psum is free once every thread has read its rows
      __syncthreads();
      if (lane == 0) wb[wave] = best;
      __syncthreads();
      if (tid == 0) {
        Best r = wb[0];
        for (int w = 1; w < SK_WAVES; ++w) if (better(wb[w], r)) r = wb[w];
        p.arg_part[(size_t)b * ARG_MAX_WG + cu] = r;
      }
    }
    cur = nxt;
    nxt = seg_desc(P, s + 2, nk, kept, cu, ncu);
  }

  // ---- greedy token: workgroup 0 reduces the per-workgroup candidates
  SK_BARRIER();
  if (cu == 0 && wave == 0) {
    Best bb{-INFINITY, 0x7fffffff};
    const Best* ap = p.arg_part + (size_t)b * ARG_MAX_WG;
    for (int i = lane; i < ncu; i += 64) { const Best c = ap[i]; if (better(c, bb)) bb = c; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const Best c{__shfl_xor(bb.v, o, 64), __shfl_xor(bb.i, o, 64)};
      if (better(c, bb)) bb = c;
    }
    if (lane == 0) {
      if (p.token_out) p.token_out[b] = bb.i;
      if (p.advance_len) p.len[b] = pos + 1;
    }
  }
#undef SK_BARRIER
}

}  // namespace first
