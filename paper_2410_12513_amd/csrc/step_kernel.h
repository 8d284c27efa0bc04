// Whole decode step of one sequence as ONE persistent kernel (bf16 models, batch 1): one 512-thread workgroup per
// compute unit.  Seven waves of a workgroup stream weights through a short ring of in-flight loads that runs on across
// phase boundaries; the eighth (the service wave) turns partial sums into outputs; all eight stage the next phase's input.  Workgroups hand activations to each other as self-validating ("tagged") words, so no
// grid barrier separates the phases.  Kept-layer indices are read from the device-side compaction, so a skipped layer
// costs neither a launch nor a byte (Section 4.3 item 2).
#pragma once
#include <type_traits>

#include "decode_kernels.h"
#include "sample_kernels.h"

namespace first {

constexpr int SK_THREADS = 512;
constexpr int SK_WAVES = SK_THREADS / 64;
constexpr int SK_SWAVES = SK_WAVES - 1;  // streaming waves; the last wave is the service wave (see k_step)
constexpr int SK_SEG = 2048;          // elements of a weight row handled by one wave at a time (4 x 16 B per lane)
// Row segments in flight per streaming wave (4 KB each).  Two - 14 MB over the chip - measured fastest on the 8B-class
// shape at 24 kept layers: 2.09 ms per step against 2.19 (one), 2.14 (three), 2.17 (four, five) and 2.18 (seven).  A deeper
// ring does not buy bandwidth, the memory system is saturated long before; it buys latency, and at every phase change the
// requests for the next phase's first rounds queue ahead of the straggling waves' last loads of this one.
constexpr int SK_PD = 2;
constexpr int SK_PSUM = 2048;         // partial sums a workgroup can hold (row segments per phase)
constexpr int SK_SMP_LISTS = 8;       // sampling in the kernel: candidate lists per lane of the merging wave (grids up to 512 workgroups)
constexpr int SK_QSPLIT_MAX = 8;      // attention of the persistent kernel: at most this many key splits per query head
constexpr unsigned SK_SPIN_LIMIT = 1u << 21;
constexpr int SK_TSLOTS = 12;         // timestamps per segment: arrive, -, attention, stage, stream, results, then six marks inside attention


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

// Activations exchanged between workgroups inside the kernel are written and read with
// device-scope (cache-coherent) accesses, so that no cache has to be flushed or invalidated:
// the L2 of each XCD is not coherent with the others for ordinary loads and stores.
__device__ __forceinline__ float ld_coh(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_coh(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned ld_coh(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coh(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coh(int* p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Batched coherent loads: request several, then wait once.  The value is defined only after
// coh_wait() followed by coh_use() on it.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void coh_issue16(f32x4_t& v, const float* p) {
  asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1" : "=v"(v) : "v"(as_global(p)) : "memory");
}
__device__ __forceinline__ void coh_issue4(float& v, const float* p) {
  asm volatile("global_load_dword %0, %1, off sc0 sc1" : "=v"(v) : "v"(as_global(p)) : "memory");
}
__device__ __forceinline__ void coh_issue4(unsigned& v, const unsigned* p) {
  asm volatile("global_load_dword %0, %1, off sc0 sc1" : "=v"(v) : "v"(as_global(p)) : "memory");
}
// Ordinary (cached) 16-byte load with the same request / wait / use protocol: where register
// pressure matters this keeps the compiler from overlapping more requests than intended.
__device__ __forceinline__ void gl_issue16(u32x4_t& v, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(as_global(reinterpret_cast<const u32x4_t*>(p))) : "memory");
}
__device__ __forceinline__ void st_coh16(float* p, const f32x4_t& v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" :: "v"(as_global(p)), "v"(v) : "memory");
}
__device__ __forceinline__ void coh_wait() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
template <typename T>
__device__ __forceinline__ void coh_use(T& v) { asm volatile("" : "+v"(v)); }

// ---------------------------------------------------------------------------------------
// Tagged exchange.  A vector that one phase produces and the next one consumes can carry its
// own "ready" signal: every 32-bit word holds the value in its upper 31 bits and, in the lowest
// mantissa bit, a tag that alternates between consecutive writes of that vector.  A consumer
// that expects tag t re-reads until every word shows t; a word is written by one aligned
// 32-bit store, so it is either the previous or the current value, never a mixture.  This
// replaces "store, wait for the store, arrive at a grid barrier, wait, load" by "store" and
// "load until current", one memory round trip instead of three or four.
//
// Why one bit is enough: a workgroup can be at most one phase ahead of the slowest one (to
// finish staging a phase's input it needs every workgroup's output of the phase before), and
// each vector is written at most once per phase, so a reader only ever meets the write it
// waits for or the one before it.  Relative error of dropping the last mantissa bit: 2^-23.
// Nothing computes on a tagged word: an infinity with tag 1 is a NaN pattern while it sits in memory and the same
// infinity again after sk_untag.
__device__ __forceinline__ float sk_tagged(float v, unsigned bit) {
  return __uint_as_float((__float_as_uint(v) & ~1u) | bit);
}
__device__ __forceinline__ float sk_untag(float v) { return __uint_as_float(__float_as_uint(v) & ~1u); }
__device__ __forceinline__ f32x4_t sk_untag(f32x4_t v) {
  v.x = sk_untag(v.x); v.y = sk_untag(v.y); v.z = sk_untag(v.z); v.w = sk_untag(v.w);
  return v;
}
// Collects the tags of the words seen so far: good(bit) iff all of them equal bit.
struct SkTags {
  unsigned any = 0u, all = ~0u;
  __device__ __forceinline__ void add(float v) { const unsigned u = __float_as_uint(v); any |= u; all &= u; }
  __device__ __forceinline__ void add(const f32x4_t& v) { add(v.x); add(v.y); add(v.z); add(v.w); }
  __device__ __forceinline__ bool good(unsigned bit) const { return bit ? (all & 1u) != 0u : (any & 1u) == 0u; }
};
// One more failed poll: gives up (and says so in *err) after the limit of polls or when another wave of the grid has
// given up; e is *err as read together with the poll.  Bit 0 of *err: somebody gave up.  The bits above it, if not zero:
// the limit + 1 for this launch instead of SK_SPIN_LIMIT - what a test writes to see the kernel give up and every wave
// leave in an orderly way, without anything having to go wrong first.
__device__ __forceinline__ bool sk_poll_give_up(unsigned& spins, int e, int* err) {
  const unsigned limit = ((unsigned)e >> 1) != 0u ? ((unsigned)e >> 1) - 1u : SK_SPIN_LIMIT;
  if (++spins <= limit && (e & 1) == 0) { __builtin_amdgcn_s_sleep(2); return false; }
  __hip_atomic_fetch_or(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return true;
}
__device__ __forceinline__ void coh_issue4(int& v, const int* p) {
  asm volatile("global_load_dword %0, %1, off sc0 sc1" : "=v"(v) : "v"(as_global(p)) : "memory");
}

// Wave-wide sum through the DPP cross-lane paths (a few cycles per step instead of an LDS
// round trip per step): quads, half rows, rows, then the two row broadcasts of gfx9.  The
// total ends up in lane 63.  Fixed order, so results are reproducible.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum_lane63(float v) {
  v = dpp_add<0xB1, 0xf>(v);     // quad_perm [1,0,3,2]
  v = dpp_add<0x4E, 0xf>(v);     // quad_perm [2,3,0,1]
  v = dpp_add<0x141, 0xf>(v);    // row_half_mirror
  v = dpp_add<0x140, 0xf>(v);    // row_mirror: every lane holds its row's sum
  v = dpp_add<0x142, 0xa>(v);    // row_bcast15 into rows 1 and 3
  v = dpp_add<0x143, 0xc>(v);    // row_bcast31 into rows 2 and 3
  return v;
}
// The first candidate of a wave in the sampling order (larger logit, then lower token index; sample_kernels.h), the same
// in every lane, through the same DPP paths: the pair travels as a 64-bit key whose unsigned order is that order.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void dpp_first(unsigned& hi, unsigned& lo) {
  const unsigned oh = (unsigned)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, ROW_MASK, 0xf, false);
  const unsigned ol = (unsigned)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, ROW_MASK, 0xf, false);
  const bool take = oh > hi || (oh == hi && ol > lo);
  hi = take ? oh : hi;
  lo = take ? ol : lo;
}
__device__ __forceinline__ Cand wave_first(const Cand& c) {
  const unsigned u = __float_as_uint(c.v + 0.0f);                       // (-0 and +0 are one logit)
  unsigned hi = u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u), lo = ~(unsigned)c.i;
  dpp_first<0xB1, 0xf>(hi, lo);      // quad_perm [1,0,3,2]
  dpp_first<0x4E, 0xf>(hi, lo);      // quad_perm [2,3,0,1]
  dpp_first<0x141, 0xf>(hi, lo);     // row_half_mirror
  dpp_first<0x140, 0xf>(hi, lo);     // row_mirror
  dpp_first<0x142, 0xa>(hi, lo);     // row_bcast15 into rows 1 and 3
  dpp_first<0x143, 0xc>(hi, lo);     // row_bcast31 into rows 2 and 3: lane 63 has seen every lane
  hi = (unsigned)__builtin_amdgcn_readlane((int)hi, 63);
  lo = (unsigned)__builtin_amdgcn_readlane((int)lo, 63);
  return Cand{__uint_as_float(hi ^ ((hi >> 31) ? 0x80000000u : 0xffffffffu)), (int)~lo};
}
// Waits until every global load and store this wave has issued is complete.
__device__ __forceinline__ void vm_wait_all() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
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
  DecParams d;                 // geometry, workspaces, sequence slot (layer fields unused); h, qkv, attn and z hold tagged words
  const LayerDev* layers;      // [L]
  const int* kept;             // [B][L] ascending kept-layer indices
  const int* n_kept;           // [B]
  int L;
  unsigned* done;              // [grid] per-workgroup "my greedy candidate is stored" epochs (never cleared: epochs only grow)
  int* err;                    // set to 1 if a wait between workgroups gives up
  int* tagstate;               // [B][8]: tags of the latest writes to the h, qkv, attn and z vectors of each slot, [4] = epoch of the
                               //         latest launch's final reduction
  float* h_out;                // [B][D] plain copy of the final hidden state (d.h holds tagged words)
  int zperm;                   // 1: the layers' down-projection matrices are the column-permuted copies (seg_blocks_gateup)
  float* part;                 // [B][Hq][SK_QSPLIT_MAX][hd + 4] tagged partial attention results of key splits 1.. (o[hd], max, sum)
  bf16 *xh_out, *xl_out;       // sk_attention<.., SPLIT_OUT> (batched path): the attention output as bf16 high / low halves in
  int out_slot;                //   A-operand order (bg_aidx) for slot out_slot, instead of fp32 in d.attn
  unsigned long long* tdbg;    // optional [segments][SK_TSLOTS] timestamps of workgroup 0 (100 MHz clock)
  // The paper's decoding rule in place of the greedy argmax (smp_k = 0: greedy; see sample_kernels.h)
  int smp_k;                   // candidates, 1 .. sk_sample_kmax(...)
  float smp_temperature;
  const float* smp_u;          // [B] the caller's uniform draws
  Cand* smp_part;              // [grid][smp_k] every workgroup's first smp_k candidates among its rows of the LM head
  int* smp_cand_out;           // [B][smp_k] the sequence's candidates in order, -1 beyond the vocabulary (may be null)
};

// LDS carve-up (floats)
struct SkLds {
  float* xs;      // [max(D, Hq*hd)] activation vector of the running phase
  float* zs;      // [F] MLP activation for the down projection
  float* psum;    // [SK_PSUM]
  float* gs;      // [min(pad(D), 4096)] RMSNorm gains of the next phase that has a norm, two-plane layout like xs
  float* red;     // [SK_WAVES + 8]
  float* qs;      // [G*hd] rotated, pre-scaled queries of this workgroup's KV head
  float* knew;    // [hd]
  float* vnew;    // [hd]
  float2* cs;     // [hd/2]
  float* ps;      // [SK_WAVES][64]
  float* mb;      // [SK_WAVES][hd + 2]
  int* flag;      // [16]: [0] verdict of the service wave's latest wait, [2] K-segments of z staged for the down projection,
                  //       [4 + w] rounds of the running phase streaming wave w has finished (gate/up in blocks)
};

__host__ __device__ inline size_t sk_lds_floats(int D, int nq, int F, int G, int hd) {
  const int xs = (D > nq ? D : nq) == 0 ? 0 : ((D > nq ? D : nq) + 2047) / 2048 * 2048;     // staged vectors are padded to whole segments
  F = (F + 2047) / 2048 * 2048;
  const int gs = ((D + 2047) / 2048 * 2048) < 4096 ? ((D + 2047) / 2048 * 2048) : 4096;
  return (size_t)xs + F + SK_PSUM + gs + (SK_WAVES + 8) + (size_t)G * hd + 2 * hd + hd + SK_WAVES * 64 +
         (size_t)SK_WAVES * (hd + 2) + 16;
}

// Largest top-k the persistent kernel can sample with on a grid of ncu workgroups: workgroup 0 merges ncu lists of k
// candidates (value + index) in the LDS that the input vectors and the partial sums occupied, plus the k it picks.
__host__ __device__ inline int sk_sample_kmax(int D, int nq, int F, int ncu) {
  const int xs = ((D > nq ? D : nq) + 2047) / 2048 * 2048;
  const long long floats = (long long)xs + (F + 2047) / 2048 * 2048 + SK_PSUM;
  const long long k = floats / (2ll * ncu + 2);
  if (ncu > 64 * SK_SMP_LISTS) return 0;
  return (int)(k < SMP_KMAX ? k : SMP_KMAX);
}

__device__ __forceinline__ SkLds sk_carve(float* base, int D, int nq, int F, int G, int hd) {
  SkLds s;
  const int xs = ((D > nq ? D : nq) + 2047) / 2048 * 2048;
  s.xs = base; base += xs;
  s.zs = base; base += (F + 2047) / 2048 * 2048;
  s.psum = base; base += SK_PSUM;
  s.gs = base; base += ((D + 2047) / 2048 * 2048) < 4096 ? ((D + 2047) / 2048 * 2048) : 4096;
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

// A staged vector of K elements occupies K rounded up to whole 2048-element segments: the
// second plane starts at sk_plane(K), and the padding of both planes is zero (a row segment
// that reaches past the end of its weight row reads zeros there, and 0 * 0 must not meet a
// stale NaN).
__host__ __device__ __forceinline__ int sk_pad(int K) { return (K + SK_SEG - 1) / SK_SEG * SK_SEG; }
__host__ __device__ __forceinline__ int sk_plane(int K) { return sk_pad(K) >> 1; }

// Zeroes the padding of both planes (nothing to do when K is a whole number of segments).
__device__ __forceinline__ void sk_zero_pad(float* xs, int K) {
  const int ngroups = K >> 3, gpad = sk_pad(K) >> 3, plane = sk_plane(K);
  if (gpad == ngroups) return;
  const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
  for (int g = ngroups + (int)(threadIdx.x & 63); g < gpad; g += 64) {
    *reinterpret_cast<f32x4_t*>(xs + (g << 2)) = zero;
    *reinterpret_cast<f32x4_t*>(xs + plane + (g << 2)) = zero;
  }
}

// A lane index the compiler cannot prove loop-invariant: address arithmetic that depends on it
// is redone (a few ALU operations) where it is used, instead of being computed once before the
// phase loop and then spilled to scratch memory for lack of registers.
__device__ __forceinline__ int sk_lane_opaque() {
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  return lane;
}

// RMSNorm gains of a vector of at most 4096 elements into LDS, in the two-plane layout of the
// staged vectors.  They are constants: the service wave fetches them while the phase before
// streams, so that nothing stands between the arrival of a phase's input and its staging.
__device__ __forceinline__ void sk_gains_to_lds(float* gs, const float* gain, int K) {
  const int lane = sk_lane_opaque(), ngroups = K >> 3, plane = sk_plane(K);
  f32x4_t a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int k = min(i * 64 + lane, ngroups - 1) << 3;
    a[i] = *as_global(reinterpret_cast<const f32x4_t*>(gain + k));
    b[i] = *as_global(reinterpret_cast<const f32x4_t*>(gain + k + 4));
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int g = i * 64 + lane;
    if (g < ngroups) {
      *reinterpret_cast<f32x4_t*>(gs + (g << 2)) = a[i];
      *reinterpret_cast<f32x4_t*>(gs + plane + (g << 2)) = b[i];
    }
  }
}

// xs <- RMSNorm(x; gains) for K <= 4096 in one pass: one batch of coherent loads, the sum of
// squares over the wave, one write of the scaled values.  Executed by the service wave.
// TAG: x holds tagged words; the batch is re-read until every word carries tag `bit`
// (returns false if that wait gives up).
template <bool TAG>
__device__ __forceinline__ bool sk_stage_norm_wave(float* xs, const float* x, int K, const float* gs, float eps,
                                                   unsigned bit, int* err) {
  const int lane = sk_lane_opaque(), ngroups = K >> 3;
  f32x4_t a[8], b[8];
  unsigned spins = 0;
  for (;;) {
    int e = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = min(i * 64 + lane, ngroups - 1) << 3;
      coh_issue16(a[i], x + k);
      coh_issue16(b[i], x + k + 4);
    }
    if (TAG) coh_issue4(e, err);
    coh_wait();
#pragma unroll
    for (int i = 0; i < 8; ++i) { coh_use(a[i]); coh_use(b[i]); }
    if (!TAG) break;
    coh_use(e);
    SkTags t;
#pragma unroll
    for (int i = 0; i < 8; ++i) { t.add(a[i]); t.add(b[i]); }
    if (__all(t.good(bit))) break;
    if (sk_poll_give_up(spins, uni(e), err)) return false;
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (TAG) { a[i] = sk_untag(a[i]); b[i] = sk_untag(b[i]); }
    if (i * 64 + lane < ngroups) {
      const f32x4_t u = a[i], v = b[i];
      ss += u.x * u.x + u.y * u.y + u.z * u.z + u.w * u.w + v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
  }
  const float r = 1.0f / sqrtf(wave_sum(ss) / (float)K + eps);
  const int plane = sk_plane(K);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int g = i * 64 + lane;
    if (g < ngroups) {
      const f32x4_t ga = *reinterpret_cast<const f32x4_t*>(gs + (g << 2));
      const f32x4_t gb = *reinterpret_cast<const f32x4_t*>(gs + plane + (g << 2));
      *reinterpret_cast<f32x4_t*>(xs + (g << 2)) = a[i] * ga * r;
      *reinterpret_cast<f32x4_t*>(xs + plane + (g << 2)) = b[i] * gb * r;
    }
  }
  sk_zero_pad(xs, K);
  return true;
}

// One wave's share of staging a normed input for K <= 4096 (gains in LDS): the groups of eight values wave * 64 + lane,
// + 512, ... .  All eight waves of the workgroup take part - between two phases the streaming waves have nothing else
// to do, and one wave alone spends most of a microsecond on the 64 values per lane that follow the poll.  The wave
// re-reads its words until they carry tag `bit`, writes gain * x into xs - NOT yet divided by the root mean square,
// which nobody knows before every wave is through - and returns its sum of squares; the phase's results are scaled
// instead (sk_norm_scale).  Returns false if the wait gives up.
__device__ __forceinline__ bool sk_stage_norm_slice(float* xs, const float* x, int K, const float* gs, unsigned bit,
                                                    int* err, int wave, float& ssq) {
  const int lane = sk_lane_opaque(), ngroups = K >> 3, plane = sk_plane(K);
  float ss = 0.f;
  unsigned spins = 0;
  for (int g0 = wave * 64; g0 < ngroups; g0 += SK_WAVES * 64) {
    const int g = g0 + lane, gc = min(g, ngroups - 1);       // (lanes past the end re-read the last group)
    f32x4_t a, b;
    for (;;) {
      int e = 0;
      coh_issue16(a, x + (gc << 3));
      coh_issue16(b, x + (gc << 3) + 4);
      coh_issue4(e, err);
      coh_wait();
      coh_use(a); coh_use(b); coh_use(e);
      SkTags t;
      t.add(a); t.add(b);
      if (__all(t.good(bit))) break;
      if (sk_poll_give_up(spins, uni(e), err)) return false;
    }
    if (g < ngroups) {
      a = sk_untag(a); b = sk_untag(b);
      ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w + b.x * b.x + b.y * b.y + b.z * b.z + b.w * b.w;
      const f32x4_t ga = *reinterpret_cast<const f32x4_t*>(gs + (g << 2));
      const f32x4_t gb = *reinterpret_cast<const f32x4_t*>(gs + plane + (g << 2));
      *reinterpret_cast<f32x4_t*>(xs + (g << 2)) = a * ga;
      *reinterpret_cast<f32x4_t*>(xs + plane + (g << 2)) = b * gb;
    }
  }
  ssq = wave_sum(ss);
  return true;
}
// The same for an input without a norm (the attention output): the wave's groups of x into xs, untagged.
__device__ __forceinline__ bool sk_stage_plain_slice(float* xs, const float* x, int K, unsigned bit, int* err, int wave) {
  const int lane = sk_lane_opaque(), ngroups = K >> 3, plane = sk_plane(K);
  unsigned spins = 0;
  for (int g0 = wave * 64; g0 < ngroups; g0 += SK_WAVES * 64) {
    const int g = g0 + lane, gc = min(g, ngroups - 1);
    f32x4_t a, b;
    for (;;) {
      int e = 0;
      coh_issue16(a, x + (gc << 3));
      coh_issue16(b, x + (gc << 3) + 4);
      coh_issue4(e, err);
      coh_wait();
      coh_use(a); coh_use(b); coh_use(e);
      SkTags t;
      t.add(a); t.add(b);
      if (__all(t.good(bit))) break;
      if (sk_poll_give_up(spins, uni(e), err)) return false;
    }
    if (g < ngroups) {
      *reinterpret_cast<f32x4_t*>(xs + (g << 2)) = sk_untag(a);
      *reinterpret_cast<f32x4_t*>(xs + plane + (g << 2)) = sk_untag(b);
    }
  }
  return true;
}
// 1 / rms of the vector the eight waves staged (their sums of squares in red[0..8), added in wave order).
__device__ __forceinline__ float sk_norm_scale(const float* red, int K, float eps) {
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < SK_WAVES; ++w) t += red[w];
  return 1.0f / sqrtf(t / (float)K + eps);
}

// xs <- x or RMSNorm(x; gain), in the two-plane layout the 8-wide weight vectors read.
// Executed by ONE wave (the service wave).  x was written by other workgroups in this
// kernel: coherent 16-byte loads, 16 requested per lane before each wait (more in flight per
// wave measured slower while the weight stream is running).  TAG as above, batch by batch.
template <bool TAG>
__device__ __forceinline__ bool sk_stage_wave(float* xs, const float* x, int K, const float* gain, float eps,
                                              unsigned bit, int* err) {
  constexpr int NB = 8;
  const int lane = sk_lane_opaque();
  const int ngroups = K >> 3, plane = sk_plane(K);
  float ss = 0.f;
  unsigned spins = 0;
  for (int g0 = 0; g0 < ngroups; g0 += NB * 64) {
    f32x4_t a[NB], b[NB];
    for (;;) {
      int e = 0;
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int k = min(g0 + i * 64 + lane, ngroups - 1) << 3;      // out-of-range groups re-read the last one
        coh_issue16(a[i], x + k);
        coh_issue16(b[i], x + k + 4);
      }
      if (TAG) coh_issue4(e, err);
      coh_wait();
#pragma unroll
      for (int i = 0; i < NB; ++i) { coh_use(a[i]); coh_use(b[i]); }
      if (!TAG) break;
      coh_use(e);
      SkTags t;
#pragma unroll
      for (int i = 0; i < NB; ++i) { t.add(a[i]); t.add(b[i]); }
      if (__all(t.good(bit))) break;
      if (sk_poll_give_up(spins, uni(e), err)) return false;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int g = g0 + i * 64 + lane;
      if (g < ngroups) {
        f32x4_t u = a[i], v = b[i];
        if (TAG) { u = sk_untag(u); v = sk_untag(v); }
        ss += u.x * u.x + u.y * u.y + u.z * u.z + u.w * u.w + v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        if (gain) {
          const f32x4_t g0v = *as_global(reinterpret_cast<const f32x4_t*>(gain + (g << 3)));
          const f32x4_t g1v = *as_global(reinterpret_cast<const f32x4_t*>(gain + (g << 3) + 4));
          u *= g0v; v *= g1v;
        }
        *reinterpret_cast<f32x4_t*>(xs + (g << 2)) = u;
        *reinterpret_cast<f32x4_t*>(xs + plane + (g << 2)) = v;
      }
    }
  }
  sk_zero_pad(xs, K);
  if (gain) {
    const float r = 1.0f / sqrtf(wave_sum(ss) / (float)K + eps);
    for (int g = lane; g < ngroups; g += 64) {                      // each lane rescales what it wrote
      f32x4_t* u = reinterpret_cast<f32x4_t*>(xs + (g << 2));
      f32x4_t* v = reinterpret_cast<f32x4_t*>(xs + plane + (g << 2));
      *u = *u * r; *v = *v * r;
    }
  }
  return true;
}

// K-segments [c0, c1) (2048 elements each, c1 - c0 <= 2) of x into the two-plane layout, no
// norm: one batch of coherent loads.  Executed by the service wave.  TAG as above.
template <bool TAG>
__device__ __forceinline__ bool sk_stage_segments(float* xs, const float* x, int K, int c0, int c1, unsigned bit, int* err) {
  const int lane = sk_lane_opaque();
  const int g_begin = c0 * (SK_SEG / 8), g_pad = c1 * (SK_SEG / 8), g_end = min(g_pad, K >> 3), plane = sk_plane(K);
  f32x4_t a[8], b[8];
  unsigned spins = 0;
  for (;;) {
    int e = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int k = min(g_begin + i * 64 + lane, g_end - 1) << 3;
      coh_issue16(a[i], x + k);
      coh_issue16(b[i], x + k + 4);
    }
    if (TAG) coh_issue4(e, err);
    coh_wait();
#pragma unroll
    for (int i = 0; i < 8; ++i) { coh_use(a[i]); coh_use(b[i]); }
    if (!TAG) break;
    coh_use(e);
    SkTags t;
#pragma unroll
    for (int i = 0; i < 8; ++i) { t.add(a[i]); t.add(b[i]); }
    if (__all(t.good(bit))) break;
    if (sk_poll_give_up(spins, uni(e), err)) return false;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int g = g_begin + i * 64 + lane;
    if (g < g_end) {
      *reinterpret_cast<f32x4_t*>(xs + (g << 2)) = TAG ? sk_untag(a[i]) : a[i];
      *reinterpret_cast<f32x4_t*>(xs + plane + (g << 2)) = TAG ? sk_untag(b[i]) : b[i];
    }
  }
  if (g_pad > g_end) sk_zero_pad(xs, K);
  return true;
}

// A segment is one mat-vec phase of the step (QKV, O, gate/up, down of a kept layer, or the
// LM head).  Rows [row0, row0+nrows) of its [N, K] matrix belong to this workgroup; a unit
// is one 2048-element piece of one row and goes to streaming wave (unit % SK_SWAVES) in round
// (unit / SK_SWAVES).  The number of rounds is padded to a multiple of SK_PD so that the ring
// of in-flight loads keeps a static register assignment across segments.
enum { SEG_QKV = 0, SEG_O = 1, SEG_GU = 2, SEG_DN = 3, SEG_HEAD = 4, SEG_NONE = 5 };
struct SegDesc {
  const bf16 *m0, *m1, *m2;     // up to three stacked matrices (or two interleaved ones)
  int n0, n1, K, inter;
  int xplane;                   // offset of the second plane of the staged input vector (sk_plane(K))
  int row0, nrows, nseg, nunits, nr_pad;
  // Unit order: the rows of a workgroup form blocks of bl rows; a block's units are ordered K-segment-major (all its rows
  // of segment 0, then of segment 1, ...) and the blocks follow each other.  One block (bl = nrows) for every phase but
  // gate/up, whose blocks are the chunks of z it produces for the down projection's K-segments (see seg_split_gateup).
  int bl, upb, blk_stride;      // rows per block, units per block (bl * nseg), distance in rows between the blocks' first rows
  unsigned inv_bl, inv_upb;     // ceil(2^32 / x): u / x = umulhi(u, inv_x) for the small u here (x <= 1 handled at use)
  int sh_bl, sh_upb;            // log2 of bl and upb when the phase runs in blocks
  int kind;
  const float* gain;            // RMSNorm gain of the phase's input (null: no norm)
  bf16* kv;                     // KV pool of the layer (attention precedes SEG_O)
};

// Rows of a phase are dealt out evenly over ncu workgroups: w0 and w1 are 1024 x (this workgroup's rank, rank + 1) among
// them (w0 = w1: no rows), which gives rows [n * rank / ncu, n * (rank + 1) / ncu).
struct SkShare { int w0, w1, ncu; };

__device__ __forceinline__ void seg_split(SegDesc& d, int N, int K, const SkShare& sh, int pair) {
  const int n = N / pair;
  d.K = K;
  d.xplane = sk_plane(K);
  // 64-bit product, 32-bit division (n * w >> 10 < 2^31 is checked on the host): 64-bit
  // division is emulated and costs dozens of registers
  d.row0 = (int)((unsigned)(((unsigned long long)(unsigned)n * (unsigned)sh.w0) >> 10) / (unsigned)sh.ncu) * pair;
  d.nrows = (int)((unsigned)(((unsigned long long)(unsigned)n * (unsigned)sh.w1) >> 10) / (unsigned)sh.ncu) * pair - d.row0;
  d.nseg = (K + SK_SEG - 1) / SK_SEG;               // the last segment of a row may be partial (reads past the row end return zeros)
  d.nunits = d.nrows * d.nseg;
  d.bl = d.nrows; d.upb = d.nunits; d.blk_stride = 0; d.sh_bl = 0; d.sh_upb = 0;
  d.inv_bl = d.bl <= 1 ? 0u : (unsigned)((0x100000000ull + d.bl - 1) / d.bl);
  d.inv_upb = d.upb <= 1 ? 0u : (unsigned)((0x100000000ull + d.upb - 1) / d.upb);
  const int nr = (d.nunits + SK_SWAVES - 1) / SK_SWAVES;
  d.nr_pad = max(SK_PD, (nr + SK_PD - 1) / SK_PD * SK_PD);
}

// Gate/up in blocks, so that z leaves in the order the down projection consumes it.  The down projection reads its input
// in K-segments of SK_SEG elements.  If every workgroup produced cs = SK_SEG / ncu elements of EVERY segment, finishing
// them segment by segment, z's first segment would be complete, grid-wide, after 1 / nseg(F) of the gate/up phase
// instead of at its end, and the down projection would never wait for its input.  Taking those elements from the
// matching rows of the gate and up matrices (stride SK_SEG between a workgroup's blocks) measured 4 us per layer slower
// than streaming one contiguous range of rows.  So the workgroup keeps its contiguous range - block k = its k-th group of
// cs rows (gate and up interleaved: 2 cs rows of the stacked numbering) - and the ORDER OF z changes instead: element i
// of block k of workgroup `rank` is z'[k * SK_SEG + cs * rank + i], and the down projection multiplies z' with a copy
// of its matrix whose columns are permuted the same way (sk_zperm_source, made once at context creation).
// Needs that copy (zperm), F to be whole segments and ncu to divide SK_SEG; otherwise one contiguous block, z in natural
// order.  Called after seg_split(d, 2 * F, K, sh, 2).
// (Written as selects between integers: a branch here makes the compiler keep the descriptor in scratch memory.)
// (D enters through the K-segments of the gate/up input: rows and units per block must be powers of two)
__host__ __device__ __forceinline__ bool sk_zperm_fits(int F, int D, int ncu) {
  const int nsegk = (D + SK_SEG - 1) / SK_SEG, cs = ncu > 0 && SK_SEG % ncu == 0 ? SK_SEG / ncu : 0;
  return F % SK_SEG == 0 && cs >= 1 && (cs & (cs - 1)) == 0 && (nsegk & (nsegk - 1)) == 0 && F / SK_SEG >= 2;
}
// Column of the caller's down-projection matrix (= natural index of z) that column j of the permuted copy holds.
__host__ __device__ __forceinline__ int sk_zperm_source(int j, int F, int ncu) {
  const int cs = SK_SEG / ncu, nblk = F / SK_SEG;
  const int k = j / SK_SEG, rem = j - k * SK_SEG, rank = rem / cs, i = rem - rank * cs;
  return cs * nblk * rank + cs * k + i;
}
__device__ __forceinline__ void seg_blocks_gateup(SegDesc& d, int F, const SkShare& sh, int zperm) {
  const bool blocked = zperm != 0 && sk_zperm_fits(F, d.K, sh.ncu) && sh.w1 - sh.w0 == 1024;
  const int cs = max(SK_SEG / sh.ncu, 1);
  const int bl = 2 * cs, upb = bl * d.nseg;
  d.bl = blocked ? bl : d.bl;
  d.upb = blocked ? upb : d.upb;
  d.blk_stride = blocked ? bl : 0;
  d.inv_bl = blocked ? (unsigned)((0x100000000ull + bl - 1) / bl) : d.inv_bl;
  d.inv_upb = blocked ? (unsigned)((0x100000000ull + upb - 1) / upb) : d.inv_upb;
  d.sh_bl = 31 - __clz(bl); d.sh_upb = 31 - __clz(upb);
}

// Unit u of a phase -> K-segment (and row of the stacked / interleaved matrices).  One block: one multiply-high.
// Blocks (gate/up): rows per block and units per block are powers of two (sk_zperm_fits), so shifts do.
__device__ __forceinline__ int seg_unit_sg(const SegDesc& d, int u, int& rl_out) {
  const int bl = uni(d.bl);
  int sg, rl;
  if (uni(d.blk_stride) != 0) {
    const int v = u & (uni(d.upb) - 1);
    sg = v >> uni(d.sh_bl);
    rl = (u >> uni(d.sh_upb)) * bl + (v & (bl - 1));      // (blocks follow each other: blk_stride = bl)
  } else {
    sg = bl <= 1 ? u : uni((int)__umulhi((unsigned)u, d.inv_bl));
    rl = u - sg * bl;
  }
  rl_out = rl;
  return sg;
}
__device__ __forceinline__ void seg_unit(const SegDesc& d, int u, int& row, int& sg) {
  int rl;
  sg = seg_unit_sg(d, u, rl);
  row = uni(d.row0) + rl;
}
// Sum over the K-segments of local row r (0 .. nrows-1 in unit order) of a finished phase or block.
__device__ __forceinline__ float seg_row_sum(const float* psum, const SegDesc& d, int r) {
  const int blk = d.blk_stride != 0 ? r >> d.sh_bl : 0;
  const int base = blk * d.upb + (r - blk * d.bl);
  float s = 0.f;
  for (int g = 0; g < d.nseg; ++g) s += psum[base + g * d.bl];
  return s;
}

__device__ __forceinline__ SegDesc seg_uniform(SegDesc d) {
  d.m0 = uni(d.m0); d.m1 = uni(d.m1); d.m2 = uni(d.m2); d.gain = uni(d.gain); d.kv = uni(d.kv);
  d.n0 = uni(d.n0); d.n1 = uni(d.n1); d.xplane = uni(d.xplane); d.K = uni(d.K); d.inter = uni(d.inter); d.row0 = uni(d.row0);
  d.nrows = uni(d.nrows); d.nseg = uni(d.nseg); d.nunits = uni(d.nunits); d.nr_pad = uni(d.nr_pad); d.kind = uni(d.kind);
  d.bl = uni(d.bl); d.upb = uni(d.upb); d.blk_stride = uni(d.blk_stride); d.inv_bl = (unsigned)uni((int)d.inv_bl); d.inv_upb = (unsigned)uni((int)d.inv_upb);
  d.sh_bl = uni(d.sh_bl); d.sh_upb = uni(d.sh_upb);
  return d;
}

// sh: this workgroup's share of the rows of every phase but the output projection, whose rows are dealt by sh_o (see k_step).
__device__ __forceinline__ SegDesc seg_desc_raw(const StepParams& P, int s, int nk, const int* kept, const SkShare& sh, const SkShare& sh_o) {
  const DecParams& p = P.d;
  const int nq = p.Hq * p.hd, nkv = p.Hkv * p.hd;
  SegDesc d{};
  d.kind = SEG_NONE;
  if (s > 4 * nk) return d;
  if (s == 4 * nk) {
    d.kind = SEG_HEAD; d.m0 = reinterpret_cast<const bf16*>(p.lm_head); d.n0 = p.V; d.gain = p.g_final;
    seg_split(d, p.V, p.D, sh, 1);
    return d;
  }
  const LayerDev lw = load_layer(P.layers, uni(kept[s >> 2]));
  d.kind = s & 3;
  d.kv = lw.kv;
  switch (d.kind) {
    case SEG_QKV:
      d.m0 = lw.wq; d.m1 = lw.wk; d.m2 = lw.wv; d.n0 = nq; d.n1 = nkv; d.gain = lw.g_attn;
      seg_split(d, nq + 2 * nkv, p.D, sh, 1);
      break;
    case SEG_O:
      d.m0 = lw.wo; d.n0 = p.D;
      seg_split(d, p.D, nq, sh_o, 1);
      break;
    case SEG_GU:
      d.m0 = lw.wg; d.m1 = lw.wu; d.inter = 1; d.gain = lw.g_mlp;
      seg_split(d, 2 * p.F, p.D, sh, 2);
      seg_blocks_gateup(d, p.F, sh, P.zperm);
      break;
    default:
      d.m0 = lw.wd; d.n0 = p.D;
      seg_split(d, p.D, p.F, sh, 1);
      break;
  }
  return d;
}

// Descriptor of segment s for this workgroup, every field in scalar registers.  Recomputed
// where needed rather than carried through the segment loop.
__device__ __forceinline__ SegDesc seg_desc(const StepParams& P, int s, int nk, const int* kept, const SkShare& sh, const SkShare& sh_o) {
  return seg_uniform(seg_desc_raw(P, s, nk, kept, sh, sh_o));
}

// Address of row r of a segment.  All inputs are wave-uniform, so the cases are scalar
// branches; the arithmetic is on integers (selects between pointers would be turned into an
// indexed table in scratch memory, and a scratch load in the request path would drain the
// ring of in-flight loads).
__device__ __forceinline__ unsigned long long seg_row_addr(const SegDesc& d, int r) {
  const unsigned long long b0 = reinterpret_cast<unsigned long long>(d.m0);
  const unsigned long long b1 = reinterpret_cast<unsigned long long>(d.m1);
  const unsigned long long b2 = reinterpret_cast<unsigned long long>(d.m2);
  const unsigned row_bytes = (unsigned)d.K * 2u;
  unsigned long long base;
  unsigned rr;
  if (d.inter) { base = (r & 1) ? b1 : b0; rr = (unsigned)r >> 1; }
  else if (r < d.n0) { base = b0; rr = (unsigned)r; }
  else if (r < d.n0 + d.n1) { base = b1; rr = (unsigned)(r - d.n0); }
  else { base = b2; rr = (unsigned)(r - d.n0 - d.n1); }
  return base + (unsigned long long)rr * row_bytes;
}

// Requests one round (4 x 16 B per lane) of a segment into a ring slot.  Branch-free: the
// row is addressed through a buffer descriptor that spans exactly that row, and a round that
// does not exist (padding, past the last segment, or disabled) uses an offset beyond the
// descriptor, for which the hardware returns zeros without touching memory.  Every call
// therefore issues exactly four loads, which lets the compiler keep exact counts of the
// loads in flight instead of draining the ring at every step.
__device__ __forceinline__ void sk_issue(const SegDesc& d, int round, bool enable, int wave, uint4 (&b)[4]) {
  // everything but the lane offset is the same for the whole wave: keep it in scalar registers
  const int u = uni(round * SK_SWAVES + wave);
  const int valid = uni((int)(enable && u < d.nunits));   // SEG_NONE has no units
  const int uu = valid ? u : 0;
  // (units of a block are ordered segment-major, so the first rounds of a one-block phase need only the first part of
  // its input vector)
  int rw, sg;
  seg_unit(d, uu, rw, sg);
  const unsigned long long ra = seg_row_addr(d, rw);
  bf16* row = reinterpret_cast<bf16*>(((unsigned long long)(unsigned)uni((int)(ra >> 32)) << 32) | (unsigned)uni((int)(unsigned)ra));
  const int row_bytes = uni(d.K * 2);
  const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(row, (short)0, row_bytes, 0x00020000);
  const int off = valid ? sg * (SK_SEG * 2) + (int)(threadIdx.x & 63) * 16 : row_bytes;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, off + j * 1024, 0, 2);   // 2 = non-temporal
    b[j] = make_uint4(v.x, v.y, v.z, v.w);
  }
}

// Dot product of one ring slot with the staged activation vector -> psum[unit].  The LDS
// reads are issued together and eight independent accumulators keep the FMA chains short:
// with two waves per SIMD there is little else to hide latency behind.
// staged / seen: for a phase whose input is staged segment by segment while it already
// streams (null otherwise): *staged = segments in LDS so far, seen = this wave's last reading.
__device__ __forceinline__ void sk_consume(const SegDesc& d, int round, int wave, const uint4 (&b)[4], const float* xs,
                                           float* psum, const int* staged, int& seen) {
  const int u = uni(round * SK_SWAVES + wave);
  const int valid = uni((int)(u < d.nunits));
  if (!valid) return;                              // padding round: the (zero) loads are accounted for, nothing to add
  const int lane = threadIdx.x & 63, K = uni(d.K);
  int rl_;
  const int sg = seg_unit_sg(d, u, rl_);
  if (staged != nullptr && sg >= seen) {
    unsigned spins = 0;
    do {
      seen = uni(__hip_atomic_load(staged, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
      if (seen <= sg) __builtin_amdgcn_s_sleep(4);
    } while (seen <= sg && ++spins < SK_SPIN_LIMIT);      // bounded; the service wave always gets there
  }
  const float* x0p = xs + ((sg * SK_SEG + lane * 8) >> 1);
  const float* x1p = x0p + uni(d.xplane);
  float4 x0[4], x1[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    x0[j] = *reinterpret_cast<const float4*>(x0p + j * 256);
    x1[j] = *reinterpret_cast<const float4*>(x1p + j * 256);
  }
  float acc[8];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint4 w = b[j];
    float e = __uint_as_float(w.x << 16) * x0[j].x, o = __uint_as_float(w.x & 0xffff0000u) * x0[j].y;
    e = fmaf(__uint_as_float(w.y << 16), x0[j].z, e); o = fmaf(__uint_as_float(w.y & 0xffff0000u), x0[j].w, o);
    e = fmaf(__uint_as_float(w.z << 16), x1[j].x, e); o = fmaf(__uint_as_float(w.z & 0xffff0000u), x1[j].y, o);
    e = fmaf(__uint_as_float(w.w << 16), x1[j].z, e); o = fmaf(__uint_as_float(w.w & 0xffff0000u), x1[j].w, o);
    acc[2 * j] = e; acc[2 * j + 1] = o;
  }
  const float tot = wave_sum_lane63(((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7])));
  if (lane == 63) psum[u] = tot;
}


// ---- Memory traffic for the attention wait.  With short contexts some workgroups have no part in attention (a quarter
// of them at 1024 keys with 32 query heads): their streaming waves hold the first rounds of the output projection and
// then wait, some ten microseconds per layer, with nothing requested and HBM nearly idle.  Such a wave touches the gate/up weights it will stream first afterwards - one 4-byte
// load per 64 bytes, a whole unit per instruction, into a register nobody reads - so that part of them is still in the L2
// or the memory-side cache by then, and waits for all its loads before it goes on (it would sit at the barrier anyway;
// and a wave's loads return in order, so nothing may be left ahead of the ring's).  Rounds [0, n) of phase d for this wave.
// SK_PF_ROUNDS per wave measured best on the 8B-class shape at 1024 keys: 2.06 ms per step against 2.09 without; 16
// rounds take a wave longer than the attention does and cost what they gain, 24 and more cost more - whatever the number
// of waiting workgroups, so the bound is one of a wave's time, not of bytes over the chip.
constexpr int SK_PF_ROUNDS = 12;
__device__ __forceinline__ void sk_prefetch(const SegDesc& d, int n, int wave) {
  unsigned sink = 0;
  const unsigned off = (unsigned)sk_lane_opaque() * 64u;
  const int row_bytes = uni(d.K * 2);
  for (int i = 0; i < n; ++i) {
    const int u = uni(i * SK_SWAVES + wave);
    if (u >= d.nunits) break;
    int rw, sg;
    seg_unit(d, u, rw, sg);
    const unsigned long long ua = seg_row_addr(d, rw) + (unsigned long long)(unsigned)(sg * (SK_SEG * 2));
    u32x4_t rs;                                    // buffer descriptor over the unit's bytes (past the row's end: zeros, no access)
    rs.x = (unsigned)uni((int)(unsigned)ua);
    rs.y = (unsigned)uni((int)(ua >> 32)) & 0xffffu;
    rs.z = (unsigned)min(SK_SEG * 2, row_bytes - sg * (SK_SEG * 2));
    rs.w = 0x00020000u;
    asm volatile("buffer_load_dword %0, %1, %2, 0 offen" : "+v"(sink) : "v"(off), "s"(rs) : "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" : "+v"(sink) : : "memory");
}

// ---------------------------------------------------------------------------------------
// Attention of workgroup (KV head g, split s): the waves = G query heads x (SK_WAVES/G) key groups,
// lane = key for the scores, lane = (key subgroup, 8-dim chunk) for the weighted values.
// NW = number of worker waves of the workgroup.
// This is the attention kernel body of the batched path's k_attn_tiles_b (the persistent kernel has its own, by query head).
template <int HD, int NW, bool SPLIT_OUT>
__device__ __forceinline__ bool sk_attention(const StepParams& P, bf16* pool, const SkLds& S, int g, int s, int nsplit,
                                             unsigned long long* stamps) {
  constexpr bool EXT = false;
  constexpr int out_tag = -1;
  const DecParams& p = P.d;
#define SK_ASTAMP(slot) do { if (stamps && threadIdx.x == 0) stamps[slot] = wall_clock64(); } while (0)
  SK_ASTAMP(6);
  constexpr int HALF = HD / 2, LPR = HD / 8, RPI = 64 / LPR;   // lanes per V row, V rows per load
  constexpr int NKL = HD / 8;                                  // 16-byte loads per key row
  const int b = p.b, G = p.G, Pg = p.P;
  const int tid = threadIdx.x, wave = uni((int)(threadIdx.x >> 6)), lane = tid & 63;
  // workers: the first G * nkg streaming waves = G query heads x nkg key groups
  const int nkg = NW / G;
  const bool worker = wave < G * nkg;
  const int hq = wave % G, kg = worker ? wave / G : nkg;       // kg == nkg: no tiles, no results
  const int pos = uni(p.len[b]), nkeys = pos + 1, tiles = (nkeys + 63) >> 6;
  const int tps = (tiles + nsplit - 1) / nsplit;
  const int t_first = s * tps, t_last = min(tiles, t_first + tps);
  const int nq = p.Hq * HD, nkv = p.Hkv * HD;
  const float* qkv = p.qkv + (size_t)b * (nq + 2 * nkv);
  const int* pt = p.page_table + (size_t)b * p.max_pages;
  const size_t head_off = (size_t)g * Pg * HD, v_off = (size_t)p.Hkv * Pg * HD;
  const bool owns_new = (pos >> 6) >= t_first && (pos >> 6) < t_last;
  const int sub = lane / LPR, dc = lane % LPR;

  // One 64-key tile, keys and values in the same layout: load i of lane (sub, dc) holds dims
  // dc*8 .. dc*8+7 of key t0 + RPI*i + sub, so every load instruction reads whole 2*HD-byte
  // rows (coalesced) and a lane ends up with the scores / weights of exactly the keys whose
  // values it will hold.  A tile is 64 / Pg whole pages (Pg = 16 on this path); their bases are
  // wave-uniform.  Pages past the sequence's last one are clamped to it (in bounds; those keys
  // get weight 0).  Explicit request / wait keeps keys and values from sharing registers.
  u32x4_t kv[NKL];
  constexpr int PPT = 4;                               // pages per tile (Pg = 16)
  const bf16* pbase[PPT];
  // page bases of a tile: the four table entries are fetched together (one wait), before the
  // explicitly ordered row requests
  auto tile_pages = [&](int t) {
    const int last_page = pos / Pg;
    int pg[PPT];
#pragma unroll
    for (int j = 0; j < PPT; ++j) pg[j] = pt[min(t * PPT + j, last_page)];
#pragma unroll
    for (int j = 0; j < PPT; ++j) pbase[j] = uni(pool + (size_t)uni(pg[j]) * p.page_elems + head_off);
  };
  auto request = [&](size_t kv_off) {
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      const int kin = RPI * i;                         // first key of this load within the tile (+ sub)
      gl_issue16(kv[i], pbase[kin / 16] + kv_off + (kin % 16) * HD + sub * HD + dc * 8);
    }
  };
  auto unpack = [](const u32x4_t w, float (&v)[8]) {
    v[0] = __uint_as_float(w.x << 16); v[1] = __uint_as_float(w.x & 0xffff0000u);
    v[2] = __uint_as_float(w.y << 16); v[3] = __uint_as_float(w.y & 0xffff0000u);
    v[4] = __uint_as_float(w.z << 16); v[5] = __uint_as_float(w.z & 0xffff0000u);
    v[6] = __uint_as_float(w.w << 16); v[7] = __uint_as_float(w.w & 0xffff0000u);
  };
  int t = t_first + kg;
  tile_pages(min(t, max(tiles - 1, 0)));            // a wave without a tile still issues (harmless) loads
  request(0);

  // this step's q (G heads), k and v of the KV head: one batch of coherent loads
  if (!EXT) {
    float q1, q2, k1, k2, vv;
    const int iq = min(tid, G * HALF - 1), hh = iq / HALF, dq = iq - hh * HALF;
    const int dk = min(tid, HALF - 1), dv = min(tid, HD - 1);
    coh_issue4(q1, qkv + (g * G + hh) * HD + dq);
    coh_issue4(q2, qkv + (g * G + hh) * HD + dq + HALF);
    coh_issue4(k1, qkv + nq + g * HD + dk);
    coh_issue4(k2, qkv + nq + g * HD + dk + HALF);
    coh_issue4(vv, qkv + nq + nkv + g * HD + dv);
    coh_wait();
    SK_ASTAMP(7);
    coh_use(q1); coh_use(q2); coh_use(k1); coh_use(k2); coh_use(vv);
    if (tid < G * HALF) {                            // rotate and pre-scale the queries
      const float2 c = S.cs[dq];
      S.qs[hh * HD + dq] = (q1 * c.x - q2 * c.y) * p.qscale;
      S.qs[hh * HD + dq + HALF] = (q2 * c.x + q1 * c.y) * p.qscale;
    }
    if (owns_new) {                                  // append the new key / value; keep the stored values in LDS
      const size_t base = (size_t)pt[pos / Pg] * p.page_elems + head_off + (size_t)(pos % Pg) * HD;
      if (tid < HALF) {
        const float2 c = S.cs[dk];
        const bf16 r1 = from_f32<bf16>(k1 * c.x - k2 * c.y), r2 = from_f32<bf16>(k2 * c.x + k1 * c.y);
        stg_bf16(pool + base + dk, r1); stg_bf16(pool + base + dk + HALF, r2);
        S.knew[dk] = to_f32(r1); S.knew[dk + HALF] = to_f32(r2);
      }
      if (tid < HD) {
        const bf16 r = from_f32<bf16>(vv);
        stg_bf16(pool + base + v_off + dv, r);
        S.vnew[dv] = to_f32(r);
      }
    }
  }
  lds_barrier();
  if (EXT) {
    SK_ASTAMP(7);
    if (uni(*S.flag) == 0) return false;
  }

  float m = -INFINITY, l = 0.f, o[8], qv[8], kn[8], vn[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    o[e] = 0.f;
    qv[e] = S.qs[hq * HD + dc * 8 + e];              // this lane's 8 dims of its head's query
    kn[e] = S.knew[dc * 8 + e];                      // ... and of the key / value appended in this step
    vn[e] = S.vnew[dc * 8 + e];                      //     (meaningful only in the workgroup that owns it)
  }

  for (; t < t_last; t += nkg) {
    const int t0 = t << 6;
    if (t != t_first + kg) { tile_pages(t); request(0); }   // (the first tile's keys were requested up front)
    coh_wait();
    float sc[NKL];
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      coh_use(kv[i]);
      float kf[8];
      unpack(kv[i], kf);
      const int key = t0 + RPI * i + sub;
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) d = fmaf(key == pos ? kn[e] : kf[e], qv[e], d);
      sc[i] = d;
    }
    request(v_off);                                  // values into the registers the keys used
    // finish the dot products across the LPR lanes that share a key, then the tile's softmax
    float mt = -INFINITY;
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
#pragma unroll
      for (int off = 1; off < LPR; off <<= 1) sc[i] += __shfl_xor(sc[i], off, 64);
      if (t0 + RPI * i + sub >= nkeys) sc[i] = -INFINITY;
      mt = fmaxf(mt, sc[i]);
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) mt = fmaxf(mt, __shfl_xor(mt, off, 64));
    const float mn = fmaxf(m, mt);
    const float corr = expf(m - mn);
    float ls = 0.f;
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      sc[i] = (t0 + RPI * i + sub < nkeys) ? expf(sc[i] - mn) : 0.f;     // sc now holds the weights
      ls += sc[i];
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) ls += __shfl_xor(ls, off, 64);
    l = l * corr + ls;
    m = mn;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] *= corr;
    coh_wait();
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      coh_use(kv[i]);
      float vf[8];
      unpack(kv[i], vf);
      const int key = t0 + RPI * i + sub;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float v = key == pos ? vn[e] : (key > pos ? 0.f : vf[e]);   // never-written slots: no NaN patterns
        o[e] = fmaf(sc[i], v, o[e]);
      }
    }
  }
  SK_ASTAMP(8);
  // fold the key subgroups: afterwards lanes 0..LPR-1 hold dims lane*8 .. lane*8+7
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] += __shfl_xor(o[e], off, 64);
  float* mb = S.mb + wave * (HD + 2);
  if (worker && lane < LPR) {
#pragma unroll
    for (int e = 0; e < 8; ++e) mb[lane * 8 + e] = o[e];
  }
  if (worker && lane == 0) { mb[HD] = m; mb[HD + 1] = l; }
  lds_barrier();
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
    st_coh(po + lane, a0);
    if (HD > 64) st_coh(po + lane + 64, a1);
    if (lane == 0) {
      float* pml = p.part_ml + (((size_t)b * p.Hq + H) * S_MAX + s) * 2;
      st_coh(pml, M); st_coh(pml + 1, den);
    }
  }
  // the last split of this KV head to finish merges all splits (in a fixed order: the result
  // does not depend on which one that is) and writes the attention output
  vm_wait_all();
  lds_barrier();
  SK_ASTAMP(9);
  if (tid == 0) {
    const unsigned old = __hip_atomic_fetch_add(p.attn_cnt + b * p.Hkv + g, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = (old == (unsigned)(nsplit - 1));
    if (last) __hip_atomic_store(p.attn_cnt + b * p.Hkv + g, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    S.flag[1] = last;
  }
  lds_barrier();
  SK_ASTAMP(10);
  if (uni(S.flag[1]) && kg == 0) {
    // lane = (split within a load, 4 dims): LPS lanes cover the head's HD dims, so one 16-byte
    // load per lane fetches SPI splits at once and up to NI * SPI splits arrive in one round trip
    constexpr int LPS = HD / 4, SPI = 64 / LPS, NI = 16;
    const int H = g * G + hq, q4 = (lane % LPS) * 4, sl = lane / LPS;
    const float* pml = p.part_ml + ((size_t)b * p.Hq + H) * S_MAX * 2;
    const float* po = p.part_o + ((size_t)b * p.Hq + H) * S_MAX * HD;
    float den = 0.f, M = -INFINITY;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    for (int b0 = 0; b0 < nsplit; b0 += NI * SPI) {
      f32x4_t o4[NI];
      float m_own, l_own;                              // lane j: maximum and sum of split j (nsplit <= 64)
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int ts = min(b0 + i * SPI + sl, nsplit - 1);
        coh_issue16(o4[i], po + ts * HD + q4);
      }
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
      const float resc = expf(M - Mb);               // 0 for the first batch (M = -inf)
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
    // fold the split groups (fixed order)
#pragma unroll
    for (int off = LPS; off < 64; off <<= 1) {
      den += __shfl_xor(den, off, 64);
      acc.x += __shfl_xor(acc.x, off, 64); acc.y += __shfl_xor(acc.y, off, 64);
      acc.z += __shfl_xor(acc.z, off, 64); acc.w += __shfl_xor(acc.w, off, 64);
    }
    float* out = p.attn + (size_t)b * nq + H * HD + q4;
    f32x4_t r = {acc.x / den, acc.y / den, acc.z / den, acc.w / den};
    if (out_tag >= 0) {
      const unsigned tb = (unsigned)out_tag;
      r.x = sk_tagged(r.x, tb); r.y = sk_tagged(r.y, tb); r.z = sk_tagged(r.z, tb); r.w = sk_tagged(r.w, tb);
    }
    if (SPLIT_OUT) {
      if (sl == 0) {
        const float v[4] = {r.x, r.y, r.z, r.w};
        unsigned short hi[4], lo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bf16 h = from_f32<bf16>(v[j]);
          hi[j] = h.v; lo[j] = from_f32<bf16>(v[j] - to_f32(h)).v;
        }
        const size_t at = bg_aidx(P.out_slot, H * HD + q4);          // 4 consecutive elements: 8 bytes, aligned
        *reinterpret_cast<uint2*>(P.xh_out + at) = make_uint2(hi[0] | ((unsigned)hi[1] << 16), hi[2] | ((unsigned)hi[3] << 16));
        *reinterpret_cast<uint2*>(P.xl_out + at) = make_uint2(lo[0] | ((unsigned)lo[1] << 16), lo[2] | ((unsigned)lo[3] << 16));
      }
    } else {
      if (sl == 0) st_coh16(out, r);
      if (out_tag < 0) vm_wait_all();
    }
  }
  SK_ASTAMP(11);
#undef SK_ASTAMP
  return true;
}

// ---------------------------------------------------------------------------------------
// Attention inside the persistent kernel.  Workgroup (query head H, key split s): its seven streaming waves take one
// 64-key tile each (more in turn when the context is long), lane = (key subgroup, 8-dim chunk); keys AND values of a
// tile are requested together, before the queries are known, so a tile costs one memory round trip.  The service wave
// fetches q of head H and k, v of its KV head as soon as they are current, rotates them, appends the new k / v to the
// cache (one of the G workgroups that share the KV head does) and afterwards folds the seven waves' partial results.
// Key split 0 of a head then collects the other splits' partial results, which arrive as tagged words like every other
// exchanged vector, and writes the head's attention output; there is no counter and no "last arriver".
// The G query heads of a KV head sit on workgroups of the same XCD (workgroup index mod Hkv), so the tiles they
// share are fetched from memory once and served to the others by that XCD's L2.
struct SkAttnGeo {
  int H, g, s, nsplit;          // query head, its KV head, this workgroup's key split, splits per head
  int pos, tiles, t_first, t_last;
  int nact;                     // streaming waves of the workgroup that take tiles (the others keep their weight ring in flight)
  bool owns_new;                // the tile that holds the new position belongs to this split
  bool appends;                 // ... and this workgroup is the one of its KV head that writes the new k / v to the cache
};

// Key splits per query head for a context of `tiles` 64-key tiles on a grid of ncu workgroups: many, so that a workgroup
// has few tiles and each of them a wave (and a SIMD) of its own - a tile is a few thousand ALU cycles of one wave.  As
// long as that still gives every tile a wave, a quarter of the grid is left out of attention: those workgroups go on
// pulling in gate/up weights meanwhile (sk_prefetch), which measured better than their help with the tiles (8B-class
// shape, 32 query heads: 6 splits 2.048 ms per step, 8 splits 2.061; 3B-class, 24 heads: 8 splits fit either way).
// tps = tiles per split.
__device__ __forceinline__ int sk_attn_splits(int tiles, int ncu, int Hq, int& tps) {
  const int smax = max(1, min(SK_QSPLIT_MAX, ncu / Hq));
  const int sfree = max(1, min(SK_QSPLIT_MAX, (ncu - ncu / 4) / Hq));
  const int tps_free = (tiles + sfree - 1) / sfree;
  tps = tps_free <= SK_SWAVES ? tps_free : (tiles + smax - 1) / smax;
  return (tiles + tps - 1) / tps;
}

__device__ __forceinline__ SkAttnGeo sk_attn_geo(const DecParams& p, int cu, int nsplit, int tps, int pos) {
  SkAttnGeo a;
  a.g = cu % p.Hkv;
  const int j = cu / p.Hkv, hl = j % p.G;
  a.s = j / p.G;
  a.H = a.g * p.G + hl;
  a.nsplit = nsplit; a.pos = pos;
  a.tiles = (pos + 64) >> 6;
  a.t_first = a.s * tps; a.t_last = min(a.tiles, a.t_first + tps);
  a.nact = min(tps, SK_SWAVES);
  a.owns_new = (pos >> 6) >= a.t_first && (pos >> 6) < a.t_last;
  a.appends = a.owns_new && hl == 0;
  return a;
}

__host__ __device__ __forceinline__ size_t sk_part_index(int Hq, int hd, int b, int H, int s) {
  return (((size_t)b * Hq + H) * SK_QSPLIT_MAX + s) * (size_t)(hd + 4);
}

// Service wave: q of head H and k, v of KV head g into LDS as soon as they carry tag `bit` (rotated; q pre-scaled; k, v
// rounded to the cache type, the values attention uses for the new position).  Returns false if the wait gives up.
template <int HD>
__device__ __forceinline__ bool sk_attn_prologue_head(const StepParams& P, bf16* pool, const SkLds& S, const SkAttnGeo& A, unsigned bit) {
  const DecParams& p = P.d;
  constexpr int HALF = HD / 2, NV = HD / 64;
  const int b = p.b, Pg = p.P, lane = sk_lane_opaque();
  const int nq = p.Hq * HD, nkv = p.Hkv * HD;
  const float* qkv = p.qkv + (size_t)b * (nq + 2 * nkv);
  const int dp = min(lane, HALF - 1);               // (HD = 64: lanes 32.. repeat the last pair)
  float q1, q2, k1, k2, vv[NV];
  unsigned spins = 0;
  for (;;) {
    int e = 0;
    coh_issue4(q1, qkv + A.H * HD + dp);
    coh_issue4(q2, qkv + A.H * HD + dp + HALF);
    coh_issue4(k1, qkv + nq + A.g * HD + dp);
    coh_issue4(k2, qkv + nq + A.g * HD + dp + HALF);
#pragma unroll
    for (int j = 0; j < NV; ++j) coh_issue4(vv[j], qkv + nq + nkv + A.g * HD + j * 64 + lane);
    coh_issue4(e, P.err);
    coh_wait();
    coh_use(e); coh_use(q1); coh_use(q2); coh_use(k1); coh_use(k2);
    SkTags t;
    t.add(q1); t.add(q2); t.add(k1); t.add(k2);
#pragma unroll
    for (int j = 0; j < NV; ++j) { coh_use(vv[j]); t.add(vv[j]); }
    if (__all(t.good(bit))) break;
    if (sk_poll_give_up(spins, uni(e), P.err)) return false;
  }
  const float2 c = S.cs[dp];
  if (lane < HALF) {
    const float a = sk_untag(q1), bq = sk_untag(q2);
    S.qs[lane] = (a * c.x - bq * c.y) * p.qscale;
    S.qs[lane + HALF] = (bq * c.x + a * c.y) * p.qscale;
  }
  if (A.owns_new) {
    const int* pt = p.page_table + (size_t)b * p.max_pages;
    const size_t head_off = (size_t)A.g * Pg * HD, v_off = (size_t)p.Hkv * Pg * HD;
    const size_t base = (size_t)pt[A.pos / Pg] * p.page_elems + head_off + (size_t)(A.pos % Pg) * HD;
    if (lane < HALF) {
      const float a = sk_untag(k1), bk = sk_untag(k2);
      const bf16 r1 = from_f32<bf16>(a * c.x - bk * c.y), r2 = from_f32<bf16>(bk * c.x + a * c.y);
      if (A.appends) { stg_bf16(pool + base + lane, r1); stg_bf16(pool + base + lane + HALF, r2); }
      S.knew[lane] = to_f32(r1); S.knew[lane + HALF] = to_f32(r2);
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int dv = j * 64 + lane;
      const bf16 r = from_f32<bf16>(sk_untag(vv[j]));
      if (A.appends) stg_bf16(pool + base + v_off + dv, r);
      S.vnew[dv] = to_f32(r);
    }
  }
  return true;
}

// Sum over the LPR (8 or 16) lanes that share a key row, through the DPP cross-lane paths; every lane of the group
// ends up with the group's sum.
template <int LPR>
__device__ __forceinline__ float sk_keyrow_sum(float v) {
  v = dpp_add<0xB1, 0xf>(v);     // quad_perm [1,0,3,2]
  v = dpp_add<0x4E, 0xf>(v);     // quad_perm [2,3,0,1]
  v = dpp_add<0x141, 0xf>(v);    // row_half_mirror: 8 lanes
  if (LPR == 16) v = dpp_add<0x140, 0xf>(v);    // row_mirror: 16 lanes
  return v;
}

// Streaming waves of an attention workgroup.  Contains two workgroup barriers: after the first the queries are in LDS
// (returns false if the service wave reported a failed wait), before the second this wave's partial result
// (o[HD], max, sum) is in S.mb[wave].  Called by waves 0..nact-1 only: the others have no tiles, keep their weight ring in
// flight instead and only take part in the two barriers (sk_attention_idle).
template <int HD>
__device__ __forceinline__ bool sk_attention_head(const StepParams& P, const bf16* pool, const SkLds& S, const SkAttnGeo& A,
                                                  unsigned long long* stamps) {
  const DecParams& p = P.d;
#define SK_ASTAMP(slot) do { if (stamps && threadIdx.x == 0) stamps[slot] = wall_clock64(); } while (0)
  SK_ASTAMP(6);
  constexpr int LPR = HD / 8, RPI = 64 / LPR;       // lanes per key row, key rows per load instruction
  constexpr int NKL = HD / 8;                       // 16-byte loads per lane and tile (keys; as many again for the values)
  constexpr int PPT = 4;                            // 16-token pages per tile
  const int Pg = p.P;
  const int wave = uni((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;
  const int pos = A.pos, nkeys = pos + 1;
  const int* pt = p.page_table + (size_t)p.b * p.max_pages;
  const size_t head_off = (size_t)A.g * Pg * HD, v_off = (size_t)p.Hkv * Pg * HD;
  const int sub = lane / LPR, dc = lane % LPR;

  // One 64-key tile: load i of lane (sub, dc) holds dims dc*8 .. dc*8+7 of key t0 + RPI*i + sub, keys and values alike,
  // so every load instruction reads whole rows and a lane ends up with the weights of exactly the keys whose values it
  // holds.  A tile is four whole pages; pages past the sequence's last one are clamped to it (in bounds; weight 0).
  // The loads are buffer loads the compiler knows as loads (one descriptor per page): it keeps them in flight across
  // the barrier and the control flow below and waits for each register where it is first read.  (Loads issued through
  // inline asm are only safe in straight-line code: at a branch the compiler may move a "value" it believes to be
  // there to another register before the load has landed.)
  u32x4_t kk[NKL], vv[NKL];
  __amdgpu_buffer_rsrc_t prs[PPT];
  const int page_bytes = (int)(p.page_elems * 2);
  const int lane_off = (int)(head_off * 2) + (sub * HD + dc * 8) * 2;
  auto tile_pages = [&](int t) {
    const int last_page = pos / Pg;
    int pg[PPT];
#pragma unroll
    for (int j = 0; j < PPT; ++j) pg[j] = pt[min(t * PPT + j, last_page)];
#pragma unroll
    for (int j = 0; j < PPT; ++j)
      prs[j] = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(uni(pool + (size_t)uni(pg[j]) * p.page_elems)), (short)0, page_bytes, 0x00020000);
  };
  auto request = [&]() {
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      const int kin = RPI * i;
      kk[i] = __builtin_amdgcn_raw_buffer_load_b128(prs[kin / 16], lane_off + (kin % 16) * HD * 2, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      const int kin = RPI * i;
      vv[i] = __builtin_amdgcn_raw_buffer_load_b128(prs[kin / 16], lane_off + (kin % 16) * HD * 2, (int)(v_off * 2), 0);
    }
  };
  auto unpack = [](const u32x4_t w, float (&v)[8]) {
    v[0] = __uint_as_float(w.x << 16); v[1] = __uint_as_float(w.x & 0xffff0000u);
    v[2] = __uint_as_float(w.y << 16); v[3] = __uint_as_float(w.y & 0xffff0000u);
    v[4] = __uint_as_float(w.z << 16); v[5] = __uint_as_float(w.z & 0xffff0000u);
    v[6] = __uint_as_float(w.w << 16); v[7] = __uint_as_float(w.w & 0xffff0000u);
  };
  float m = -INFINITY, l = 0.f, o[8], qv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = 0.f;
  // One tile whose loads are in flight.  EDGE: the sequence's last tile, which holds the slot of the new position (its
  // key and value are taken from LDS afterwards: the cache write may not have landed) and possibly slots beyond it
  // (never written): all of those get weight 0 and their contents never enter a sum (no NaN patterns).
  // live = false: a wave beyond the split's last tile fetched an existing tile and ignores it.
  auto tile = [&](int t, bool live, auto edge_tag) {
    constexpr bool EDGE = decltype(edge_tag)::value;
    const int t0 = t << 6;
    float sc[NKL];
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      float kf[8];
      unpack(kk[i], kf);
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) d = fmaf(kf[e], qv[e], d);
      sc[i] = d;
    }
    float mt = -INFINITY;
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      sc[i] = sk_keyrow_sum<LPR>(sc[i]);
      if (EDGE && t0 + RPI * i + sub >= pos) sc[i] = -INFINITY;
      mt = fmaxf(mt, sc[i]);
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) mt = fmaxf(mt, __shfl_xor(mt, off, 64));
    // (an edge tile may hold no stored key at all: then nothing changes)
    const bool any = live && mt > -INFINITY;
    const float mn = any ? fmaxf(m, mt) : m;
    const float corr = any ? expf(m - mn) : 1.f;
    float ls = 0.f;
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      sc[i] = (any && (!EDGE || t0 + RPI * i + sub < pos)) ? expf(sc[i] - mn) : 0.f;     // sc now holds the weights
      ls += sc[i];
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) ls += __shfl_xor(ls, off, 64);
    l = l * corr + ls;
    m = mn;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] *= corr;
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      float vf[8];
      unpack(vv[i], vf);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float v = (EDGE && t0 + RPI * i + sub >= pos) ? 0.f : vf[e];
        o[e] = fmaf(sc[i], v, o[e]);
      }
    }
    if (EDGE && live) {
      // the new position: key and value as stored (rounded to the cache type), from LDS; one more key of this wave
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) d = fmaf(S.knew[dc * 8 + e], qv[e], d);
      d = sk_keyrow_sum<LPR>(d);
      const float mn2 = fmaxf(m, d);
      const float c2 = expf(m - mn2), w = expf(d - mn2);      // (m = -inf: c2 = 0)
      l = l * c2 + w;
      m = mn2;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = fmaf(sub == 0 ? w : 0.f, S.vnew[dc * 8 + e], o[e] * c2);   // (the subgroups are summed below: once)
    }
  };
  auto tile_any = [&](int t, bool live) {
    if (t == (pos >> 6)) tile(t, live, std::true_type{});
    else tile(t, live, std::false_type{});
  };

  int t = A.t_first + wave;
  const bool live0 = t < A.t_last;
  const int tfirst = live0 ? t : A.t_first;
  tile_pages(tfirst);
  request();
  lds_barrier();                                   // q, new k / v and the verdict of the service wave's wait are in LDS
  SK_ASTAMP(7);
  if (uni(*S.flag) == 0) return false;
#pragma unroll
  for (int e = 0; e < 8; ++e) qv[e] = S.qs[dc * 8 + e];     // this lane's 8 dims of the head's query
  tile_any(tfirst, live0);
  for (t += SK_SWAVES; t < A.t_last; t += SK_SWAVES) {
    tile_pages(t);
    request();
    tile_any(t, true);
  }
  SK_ASTAMP(8);
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
  lds_barrier();                                   // the service wave folds the waves' results
#undef SK_ASTAMP
  return true;
}

// A streaming wave without tiles: keeps step with the two barriers of sk_attention_head.
__device__ __forceinline__ bool sk_attention_idle(const SkLds& S) {
  lds_barrier();
  const bool ok = uni(*S.flag) != 0;
  if (ok) lds_barrier();
  return ok;
}

// Service wave, after the second barrier: folds the streaming waves' results in wave order; a split other than 0 leaves
// its result as tagged words for split 0, which waits for them (tag `bit`), folds them in split order and writes the
// head's attention output as tagged words.  Returns false if that wait gives up.
template <int HD>
__device__ __forceinline__ bool sk_attn_merge_head(const StepParams& P, const SkLds& S, const SkAttnGeo& A, unsigned bit,
                                                   unsigned long long* stamps) {
  const DecParams& p = P.d;
  constexpr int NV = HD / 64;
  const int lane = sk_lane_opaque();
  float M = -INFINITY;
  for (int w = 0; w < A.nact; ++w) M = fmaxf(M, S.mb[w * (HD + 2) + HD]);
  float den = 0.f, a[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) a[j] = 0.f;
  for (int w = 0; w < A.nact; ++w) {
    const float* src = S.mb + w * (HD + 2);
    const float lt = src[HD + 1];
    if (lt > 0.f) {
      const float wg = expf(src[HD] - M);
      den = fmaf(lt, wg, den);
#pragma unroll
      for (int j = 0; j < NV; ++j) a[j] = fmaf(src[j * 64 + lane], wg, a[j]);
    }
  }
  if (stamps && lane == 0) stamps[9] = wall_clock64();
  if (A.s != 0) {
    float* dst = P.part + sk_part_index(p.Hq, HD, p.b, A.H, A.s);
#pragma unroll
    for (int j = 0; j < NV; ++j) st_coh(dst + j * 64 + lane, sk_tagged(a[j], bit));
    if (lane < 2) st_coh(dst + HD + lane, sk_tagged(lane == 0 ? M : den, bit));
    return true;
  }
  if (A.nsplit > 1) {
    float po[SK_QSPLIT_MAX - 1][NV], pm[SK_QSPLIT_MAX - 1], pl[SK_QSPLIT_MAX - 1];
    unsigned spins = 0;
    for (;;) {
      int e = 0;
#pragma unroll
      for (int q = 0; q < SK_QSPLIT_MAX - 1; ++q) {
        const float* src = P.part + sk_part_index(p.Hq, HD, p.b, A.H, min(q + 1, A.nsplit - 1));
#pragma unroll
        for (int j = 0; j < NV; ++j) coh_issue4(po[q][j], src + j * 64 + lane);
        coh_issue4(pm[q], src + HD);
        coh_issue4(pl[q], src + HD + 1);
      }
      coh_issue4(e, P.err);
      coh_wait();
      coh_use(e);
      SkTags t;
#pragma unroll
      for (int q = 0; q < SK_QSPLIT_MAX - 1; ++q) {
#pragma unroll
        for (int j = 0; j < NV; ++j) { coh_use(po[q][j]); t.add(po[q][j]); }
        coh_use(pm[q]); coh_use(pl[q]);
        t.add(pm[q]); t.add(pl[q]);
      }
      if (__all(t.good(bit))) break;
      if (sk_poll_give_up(spins, uni(e), P.err)) return false;
    }
    if (stamps && lane == 0) stamps[10] = wall_clock64();
    float M2 = M;
#pragma unroll
    for (int q = 0; q < SK_QSPLIT_MAX - 1; ++q) {
      pm[q] = sk_untag(pm[q]); pl[q] = sk_untag(pl[q]);       // (untagging restores an infinite maximum exactly)
      if (q + 1 < A.nsplit && pl[q] > 0.f) M2 = fmaxf(M2, pm[q]);
    }
    const float f0 = den > 0.f ? expf(M - M2) : 0.f;
    den *= f0;
#pragma unroll
    for (int j = 0; j < NV; ++j) a[j] *= f0;
#pragma unroll
    for (int q = 0; q < SK_QSPLIT_MAX - 1; ++q) {
      if (q + 1 < A.nsplit && pl[q] > 0.f) {
        const float wg = expf(pm[q] - M2);
        den = fmaf(pl[q], wg, den);
#pragma unroll
        for (int j = 0; j < NV; ++j) a[j] = fmaf(sk_untag(po[q][j]), wg, a[j]);
      }
    }
  }
  float* out = p.attn + (size_t)p.b * p.Hq * HD + A.H * HD;
#pragma unroll
  for (int j = 0; j < NV; ++j) st_coh(out + j * 64 + lane, sk_tagged(a[j] / den, bit));
  if (stamps && lane == 0) stamps[11] = wall_clock64();
  return true;
}

// dst[r][j] = src[r][sk_zperm_source(j)]: the down-projection matrix with its columns in the order in which the blocked
// gate/up phase produces z (made once per layer at context creation).  Groups of SK_SEG / ncu columns move together.
__global__ void __launch_bounds__(WG) k_permute_down_columns(const bf16* __restrict__ src, bf16* __restrict__ dst, int D, int F, int ncu) {
  const int cs = SK_SEG / ncu;
  const size_t groups = (size_t)D * (F / cs);
  for (size_t g = (size_t)blockIdx.x * WG + threadIdx.x; g < groups; g += (size_t)gridDim.x * WG) {
    const size_t r = g / (F / cs);
    const int j = (int)(g - r * (F / cs)) * cs;
    const bf16* in = src + r * F + sk_zperm_source(j, F, ncu);
    bf16* out = dst + r * F + j;
    if (cs % 8 == 0) {
      for (int i = 0; i < cs; i += 8) *reinterpret_cast<uint4*>(out + i) = *reinterpret_cast<const uint4*>(in + i);
    } else {
      for (int i = 0; i < cs; ++i) out[i] = in[i];
    }
  }
}

// ---------------------------------------------------------------------------------------
// Wave roles.  Waves 0..SK_SWAVES-1 only stream weights: each keeps a ring of SK_PD rounds (8 KB) in flight that runs
// on across phase boundaries, so HBM stays busy while the workgroups hand their results on.  The last wave is the
// service wave: it turns the partial sums of a finished phase into its outputs, waits for the next phase's input and
// stages it into LDS.  It never has weight loads in flight, which matters because a wave's loads return in order: a
// poll or an input load issued behind a prefetch queue would wait for all of it.
//
// Who does what in the attention + output-projection phase.  The first Hq x nsplit workgroups compute attention (their
// tile waves have no weight loads in flight meanwhile: the ring registers hold the key and value tiles), the others touch
// gate/up weights ahead (sk_prefetch); the output projection's rows are dealt evenly over all of them, like every other
// phase's.  (Keeping its rows off the attention workgroups when those are at most half the grid - so that the others
// could hold them ready - was worth something with a deep ring; with two rounds in flight it measured 0.7 to 2 % slower
// at contexts below 200 keys, where it applied, and is gone.)
//
// The residual rows a workgroup updates in the output and down projections are fetched by its service wave right
// after it has staged the phase before (QKV or gate/up), when it has seen every word of h current.
template <int HD>
__global__ void __launch_bounds__(SK_THREADS) k_step(StepParams P) {
  extern __shared__ __align__(16) float smem_f[];
  const DecParams& p = P.d;
  const int cu = blockIdx.x, ncu = gridDim.x, tid = threadIdx.x, wave = uni((int)(threadIdx.x >> 6)), lane = tid & 63;
  const bool service = wave == SK_SWAVES;
  const int b = p.b, D = p.D, F = p.F, nq = p.Hq * HD, nkv = p.Hkv * HD;
  const SkLds S = sk_carve(smem_f, D, nq, F, p.G, HD);
  float* h = p.h + (size_t)b * D;
  // tags of the latest writes of h, qkv, attn (and the attention partials) and z: the same in every wave of the grid,
  // each flips when the phase that writes the vector begins
  // (everything a workgroup has to read before it can start is requested together: one memory round trip)
  unsigned tag_h, tag_q, tag_a, tag_z, epoch;
  int nk, pos, tok;
  {
    const int ts_v = ld_coh(P.tagstate + 8 * b + (lane & 7));      // lane l: word l of the slot's exchange state
    const int nk_v = P.n_kept[b], pos_v = p.len[b], tok_v = p.tokens[b];
    tag_h = (unsigned)__builtin_amdgcn_readlane(ts_v, 0) & 1u; tag_q = (unsigned)__builtin_amdgcn_readlane(ts_v, 1) & 1u;
    tag_a = (unsigned)__builtin_amdgcn_readlane(ts_v, 2) & 1u; tag_z = (unsigned)__builtin_amdgcn_readlane(ts_v, 3) & 1u;
    epoch = (unsigned)__builtin_amdgcn_readlane(ts_v, 4) + 1u;
    nk = uni(nk_v); pos = uni(pos_v); tok = uni(tok_v);
  }
  const int* kept = P.kept + (size_t)b * P.L;
  // attention: workgroup = (query head, key split), one 64-key tile per streaming wave where the grid allows
  const int tiles = (pos + 64) >> 6;
  int tps;
  const int nsplit = sk_attn_splits(tiles, ncu, p.Hq, tps);
  const int n_attn = p.Hq * nsplit;
  const bool attn_wg = cu < n_attn;
  const SkAttnGeo A = sk_attn_geo(p, attn_wg ? cu : 0, nsplit, tps, pos);
  const SkShare share{cu * 1024, (cu + 1) * 1024, ncu};
  const SkShare share_o = share;                   // (the output projection's rows: dealt like all others)

#define SK_STAMP(slot)                                                                 \
  do {                                                                                 \
    if (P.tdbg && cu == 0 && tid == SK_SWAVES * 64) P.tdbg[s * SK_TSLOTS + (slot)] = wall_clock64(); \
  } while (0)

  // ---- h = E[token]; rotation table of this position (kept in LDS for the whole step)
  {
    tok = min(max(tok, 0), p.V - 1);
    const bf16* row = reinterpret_cast<const bf16*>(p.embed) + (size_t)tok * D;
    SegDesc e{};
    seg_split(e, D, D, share, 1);                  // the rows this workgroup owns in the phases that write h (at most 64, checked on the host)
    tag_h ^= 1u;
    if (service && lane < e.nrows) {
      const float v = sk_untag(to_f32(row[e.row0 + lane]));
      st_coh(h + e.row0 + lane, sk_tagged(v, tag_h));
      if (P.h_out != nullptr) P.h_out[(size_t)b * D + e.row0 + lane] = v;
    }
    // a key split other than 0 leaves "not yet" (the tag of the write before) in its slot of the attention partials:
    // the slot may never have been used, or not since the context was shorter, and then carries the tag of some older write
    if (service && attn_wg && A.s != 0) {
      float* dst = P.part + sk_part_index(p.Hq, HD, b, A.H, A.s);
      for (int i = lane; i < HD + 2; i += 64) st_coh(dst + i, sk_tagged(0.f, tag_a));
      // (this wave waits for all its memory operations many times before it stores the slot's first real contents)
    }
    for (int i = tid; i < HD / 2; i += SK_THREADS) {
      const double a = (double)pos * p.theta[i];
      S.cs[i] = make_float2((float)cos(a), (float)sin(a));
    }
  }

  const int nsegs = 4 * nk + 1;

  // The two roles run separate loops (so that the service wave carries no ring registers and the streaming waves no
  // staging registers) with the same sequence of workgroup barriers.
  if (service) {
    if (lane == 0) { S.flag[12] = 1; S.flag[13] = 1; }      // verdicts of the streaming waves' shares of staging, by phase parity
    // RMSNorm gains of the next phase that has a norm: constants, fetched while the phase before streams so that they
    // are not in the way when the phase's input arrives.  Those of the first phase: before the barrier, because every
    // wave of the workgroup reads them as soon as it is past it (sk_stage_norm_slice).
    {
      const SegDesc first = seg_desc(P, 0, nk, kept, share, share_o);
      if (first.gain != nullptr && D <= 4096) sk_gains_to_lds(S.gs, first.gain, D);
    }
    lds_barrier();                                 // the rotation table and the first gains are in LDS
    float h_prev = 0.f;                            // lane r: residual row row0 + r of the coming output / down projection (tagged word)
    int z_staged = 0;                              // K-segments of the coming down projection's input already in LDS
    // (a phase's descriptor is worked out while the phase before streams: nothing but the wait for the input and its
    // staging stands between a phase's results and the next phase)
    SegDesc cur = seg_desc(P, 0, nk, kept, share, share_o);
    for (int s = 0; s < nsegs; ++s) {
      SK_STAMP(0);
      SK_STAMP(1);
      const bool fast_norm = cur.gain != nullptr && D <= 4096;
      bool staged_ok = true;
      if (cur.kind == SEG_O) {
        tag_a ^= 1u;
        if (attn_wg) {
          unsigned long long* stamps = (P.tdbg && cu == 0) ? P.tdbg + s * SK_TSLOTS : nullptr;
          const bool ok = sk_attn_prologue_head<HD>(P, cur.kv, S, A, tag_q);
          if (lane == 0) *S.flag = ok ? 1 : 0;
          lds_barrier();                           // queries in LDS, verdict visible
          if (!ok) return;
          lds_barrier();                           // the streaming waves' partial results are in LDS
          staged_ok = sk_attn_merge_head<HD>(P, S, A, tag_a, stamps);
        }
        SK_STAMP(2);
        if (cur.nrows > 0) {                       // (a share of it, like every wave of the workgroup)
          staged_ok = sk_stage_plain_slice(S.xs, p.attn + (size_t)b * nq, nq, tag_a, P.err, wave) && staged_ok;
          sk_zero_pad(S.xs, nq);
        }
      } else if (cur.kind == SEG_DN) {
        // the down projection starts on the first K-segment of its input (already staged during gate/up when that ran
        // in blocks); the rest is staged while it streams (after the workgroup barrier below)
        if (z_staged == 0) {
          staged_ok = sk_stage_segments<true>(S.zs, p.z + (size_t)b * F, F, 0, 1, tag_z, P.err);
          z_staged = 1;
          __hip_atomic_store(S.flag + 2, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
      } else if (fast_norm) {
        // (every wave of the workgroup stages a share: see sk_stage_norm_slice; the streaming waves report to flag[12 + parity])
        float ssq = 0.f;
        staged_ok = sk_stage_norm_slice(S.xs, h, D, S.gs, tag_h, P.err, wave, ssq);
        if (lane == 0) S.red[wave] = ssq;
        sk_zero_pad(S.xs, D);
      } else {
        staged_ok = sk_stage_wave<true>(S.xs, h, D, cur.gain, p.eps, tag_h, P.err);
      }
      if (lane == 0) *S.flag = staged_ok ? 1 : 0;
      if (cur.kind == SEG_GU && lane < SK_WAVES) S.flag[4 + lane] = 0;     // (rounds finished: counted from the barrier below)
      SK_STAMP(3);
      lds_barrier();                               // input vector staged; verdict of the wait visible
      if (!staged_ok || uni(S.flag[12 + (s & 1)]) == 0) return;
      if (lane == 0) S.flag[12 + ((s + 1) & 1)] = 1;       // (the next phase's word: nobody looks at it before the next barrier but one)
      // a normed input staged by all waves still lacks its 1 / rms: the phase's results are scaled by it
      const float rs = fast_norm ? sk_norm_scale(S.red, D, p.eps) : 1.0f;
      const SegDesc nx = seg_desc(P, s + 1, nk, kept, share, share_o);
      if (cur.kind == SEG_QKV || cur.kind == SEG_GU) {
        // every word of h has just been seen current: fetch the rows the next phase of this workgroup adds to
        h_prev = ld_coh(h + nx.row0 + min(lane, max(nx.nrows - 1, 0)));
      }
      if (cur.kind == SEG_DN) {
        for (int c = z_staged; c < cur.nseg; c += 2) {
          const int c1 = min(c + 2, cur.nseg);
          // (a wait that gives up has said so in *P.err: the next phase's wait ends the workgroup)
          sk_stage_segments<true>(S.zs, p.z + (size_t)b * F, F, c, c1, tag_z, P.err);
          __hip_atomic_store(S.flag + 2, c1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        z_staged = 0;
      }
      if (cur.kind == SEG_GU && cur.blk_stride != 0) {
        // Gate/up in blocks: block k is this workgroup's part of K-segment k of the down projection's input.  As soon
        // as the streaming waves are through a block its z values go out, and the segment before it - by now complete
        // grid-wide - is staged for the down projection, which therefore starts without waiting for anybody.
        float* z = p.z + (size_t)b * F;
        tag_z ^= 1u;
        const int nblk = cur.nunits / cur.upb, cs = cur.bl >> 1;
        for (int k = 0; k < nblk; ++k) {
          const int need = (k + 1) * cur.upb;          // every unit below this one has been consumed
          unsigned spins = 0;
          for (;;) {
            const int done = __hip_atomic_load(S.flag + 4 + min(lane, SK_SWAVES - 1), __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (__all(done * SK_SWAVES + min(lane, SK_SWAVES - 1) >= need) || ++spins > SK_SPIN_LIMIT) break;
            __builtin_amdgcn_s_sleep(8);
          }
          for (int r = lane; r < cs; r += 64) {
            const float gt = seg_row_sum(S.psum, cur, k * cur.bl + 2 * r) * rs, up = seg_row_sum(S.psum, cur, k * cur.bl + 2 * r + 1) * rs;
            st_coh(z + k * SK_SEG + cs * cu + r, sk_tagged(siluf(gt) * up, tag_z));
          }
          if (k >= 1 && k + 1 < nblk) {               // (not behind the last block: the down projection is waiting for this wave)
            // (a wait that gives up has said so in *P.err: the next phase's wait ends the workgroup)
            sk_stage_segments<true>(S.zs, z, F, k - 1, k, tag_z, P.err);
            z_staged = k;
            __hip_atomic_store(S.flag + 2, k, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
          }
        }
      }
      if (s + 1 < nsegs && D <= 4096 && nx.gain != nullptr) sk_gains_to_lds(S.gs, nx.gain, D);   // (this phase's staging has read S.gs already)
      lds_barrier();                               // partial sums complete
      SK_STAMP(4);
      // results of the segment
      if (cur.kind == SEG_QKV) {
        float* out = p.qkv + (size_t)b * (nq + 2 * nkv);
        tag_q ^= 1u;
        for (int r = lane; r < cur.nrows; r += 64) {
          const float v = seg_row_sum(S.psum, cur, r) * rs;
          st_coh(out + cur.row0 + r, sk_tagged(v, tag_q));
        }
      } else if (cur.kind == SEG_O || cur.kind == SEG_DN) {
        tag_h ^= 1u;
        if (lane < cur.nrows) {
          const float v = sk_untag(sk_untag(h_prev) + seg_row_sum(S.psum, cur, lane));
          st_coh(h + cur.row0 + lane, sk_tagged(v, tag_h));
          if (cur.kind == SEG_DN && P.h_out != nullptr) P.h_out[(size_t)b * D + cur.row0 + lane] = v;
        }
      } else if (cur.kind == SEG_GU && cur.blk_stride == 0) {
        float* z = p.z + (size_t)b * F;
        tag_z ^= 1u;
        for (int r = lane; r < cur.nrows / 2; r += 64) {
          const float gt = seg_row_sum(S.psum, cur, 2 * r) * rs, up = seg_row_sum(S.psum, cur, 2 * r + 1) * rs;
          st_coh(z + cur.row0 / 2 + r, sk_tagged(siluf(gt) * up, tag_z));
        }
      } else if (cur.kind == SEG_HEAD) {
        float* lg = p.logits ? p.logits + (size_t)b * p.V : nullptr;
        if (P.smp_k > 0) {
          // Sampling: this workgroup's first smp_k candidates in the order (larger logit, lower index), by smp_k rounds
          // of "first after the previous pick" over its logits, which wait in LDS (the input vector's place: the head
          // has streamed).  Workgroup 0 merges the lists the same way below.
          float* lv = S.xs;
          for (int r = lane; r < cur.nrows; r += 64) {
            const float v = seg_row_sum(S.psum, cur, r) * rs;
            if (lg) lg[cur.row0 + r] = v;
            lv[r] = v;
          }
          Cand last{INFINITY, -1};
          Cand* dst = P.smp_part + (size_t)cu * P.smp_k;
          for (int k = 0; k < P.smp_k; ++k) {
            Cand first{-INFINITY, SMP_NONE};
            for (int r = lane; r < cur.nrows; r += 64) {
              const Cand e{lv[r], cur.row0 + r};
              if (cand_before(last, e) && cand_before(e, first)) first = e;
            }
            first = wave_first(first);
            if (lane == 0) { st_coh(&dst[k].v, first.v); st_coh(&dst[k].i, first.i); }
            last = first.i == SMP_NONE ? Cand{-INFINITY, SMP_NONE} : first;      // nothing left: nothing comes after
          }
          vm_wait_all();                           // the candidates are in memory before this workgroup says so
        } else {
        Best best{-INFINITY, 0x7fffffff};
        for (int r = lane; r < cur.nrows; r += 64) {
          const float v = seg_row_sum(S.psum, cur, r) * rs;
          if (lg) lg[cur.row0 + r] = v;
          const Best c{v, cur.row0 + r};
          if (better(c, best)) best = c;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
          const Best c{__shfl_xor(best.v, o, 64), __shfl_xor(best.i, o, 64)};
          if (better(c, best)) best = c;
        }
        if (lane == 0) {
          Best* dst = p.arg_part + (size_t)b * ARG_MAX_WG + cu;
          st_coh(&dst->v, best.v); st_coh(&dst->i, best.i);
        }
        vm_wait_all();                             // the candidate is in memory before this workgroup says so
        }
      }
      SK_STAMP(5);
      cur = nx;
    }
    // greedy token: every workgroup publishes the launch's epoch once its candidate is stored; workgroup 0 waits for
    // all of them and reduces.  Epochs only grow from launch to launch, so nothing is cleared in between.
    if (lane == 0) __hip_atomic_store(P.done + cu, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (cu != 0) return;
    {
      unsigned spins = 0;
      for (;;) {
        bool ok = true;
        int e = 0;
        for (int base = 0; base < ncu; base += 256) {
          unsigned f[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) coh_issue4(f[i], P.done + min(base + i * 64 + lane, ncu - 1));
          coh_issue4(e, P.err);
          coh_wait();
          coh_use(e);
#pragma unroll
          for (int i = 0; i < 4; ++i) { coh_use(f[i]); ok = ok && (f[i] == epoch); }
        }
        if (__all(ok)) break;
        if (sk_poll_give_up(spins, uni(e), P.err)) return;
      }
    }
    Best bb{-INFINITY, 0x7fffffff};
    if (P.smp_k > 0) {
      // all candidate lists into LDS (from the input vector's place on: nothing there is needed any more; the host
      // checked that they fit), smp_k rounds over them, the draw by one lane
      const int n = ncu * P.smp_k;
      float* cv = S.xs;
      int* ci = reinterpret_cast<int*>(S.xs) + n;
      // (two candidates per 16-byte load, sixteen loads per lane in flight: one memory round trip per 2048 candidates;
      // the list buffer has SMP_KMAX slots per workgroup, so the odd one past the end is there to be read and ignored)
      const float* src = reinterpret_cast<const float*>(P.smp_part);
      for (int j0 = 0; j0 < n; j0 += 2 * 64 * 16) {
        f32x4_t q[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) coh_issue16(q[t], src + 2 * min(j0 + 2 * (t * 64 + lane), n - 1 + (n & 1) - 1));
        coh_wait();
#pragma unroll
        for (int t = 0; t < 16; ++t) {
          coh_use(q[t]);
          const int j = j0 + 2 * (t * 64 + lane);
          if (j < n) { cv[j] = q[t].x; ci[j] = __float_as_int(q[t].y); }
          if (j + 1 < n) { cv[j + 1] = q[t].z; ci[j + 1] = __float_as_int(q[t].w); }
        }
      }
      Cand* top = reinterpret_cast<Cand*>(ci + n);
      // every list is in order already, so only the lists' heads compete: a lane looks after the lists of workgroups
      // lane, lane + 64, ... (at most SK_SMP_LISTS of them: the host checks the grid), the winner's list moves on
      Cand head[SK_SMP_LISTS];
      int at[SK_SMP_LISTS];
#pragma unroll
      for (int l = 0; l < SK_SMP_LISTS; ++l) {
        const int wg = l * 64 + lane;
        at[l] = wg * P.smp_k;
        head[l] = wg < ncu ? Cand{cv[at[l]], ci[at[l]]} : Cand{-INFINITY, SMP_NONE};
      }
      for (int k = 0; k < P.smp_k; ++k) {
        Cand first{-INFINITY, SMP_NONE};
#pragma unroll
        for (int l = 0; l < SK_SMP_LISTS; ++l)
          if (head[l].i != SMP_NONE && cand_before(head[l], first)) first = head[l];
        first = wave_first(first);
        if (lane == 0) top[k] = first;
#pragma unroll
        for (int l = 0; l < SK_SMP_LISTS; ++l)
          if (head[l].i == first.i && first.i != SMP_NONE) {       // (token ids are unique: this is the list it came from)
            ++at[l];
            head[l] = at[l] < (l * 64 + lane + 1) * P.smp_k ? Cand{cv[at[l]], ci[at[l]]} : Cand{-INFINITY, SMP_NONE};
          }
      }
      if (P.smp_cand_out != nullptr)
        for (int k = lane; k < P.smp_k; k += 64) P.smp_cand_out[(size_t)b * P.smp_k + k] = top[k].i == SMP_NONE ? -1 : top[k].i;
      if (lane == 0) bb.i = smp_draw(top, P.smp_k, P.smp_temperature, P.smp_u[b]);
    } else {
    const Best* ap = p.arg_part + (size_t)b * ARG_MAX_WG;
    for (int i = lane; i < ncu; i += 64) { const Best c{ld_coh(&ap[i].v), ld_coh(&ap[i].i)}; if (better(c, bb)) bb = c; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const Best c{__shfl_xor(bb.v, o, 64), __shfl_xor(bb.i, o, 64)};
      if (better(c, bb)) bb = c;
    }
    }
    if (lane == 0) {
      if (p.token_out) p.token_out[b] = bb.i;
      if (p.advance_len) p.len[b] = pos + 1;
      int* ts = P.tagstate + 8 * b;
      st_coh(ts, (int)tag_h); st_coh(ts + 1, (int)tag_q); st_coh(ts + 2, (int)tag_a); st_coh(ts + 3, (int)tag_z);
      st_coh(ts + 4, (int)epoch);
    }
  } else {
    uint4 buf[SK_PD][4];
    {
      const SegDesc first = seg_desc(P, 0, nk, kept, share, share_o);
#pragma unroll
      for (int j = 0; j < SK_PD; ++j) sk_issue(first, j, true, wave, buf[j]);
    }
    lds_barrier();
    SegDesc cur = seg_desc(P, 0, nk, kept, share, share_o);
    for (int s = 0; s < nsegs; ++s) {
      const float* xsrc = cur.kind == SEG_DN ? S.zs : S.xs;
      if (cur.kind == SEG_O) tag_a ^= 1u;          // (as the service wave does: the tag the attention output will carry)
      if (cur.kind == SEG_O && attn_wg) {
        // (a wave that takes tiles has nothing of the ring in flight here: its registers hold the keys and values)
        unsigned long long* stamps = (P.tdbg && cu == 0) ? P.tdbg + s * SK_TSLOTS : nullptr;
        if (wave < A.nact) {
          if (!sk_attention_head<HD>(P, cur.kv, S, A, stamps)) return;
#pragma unroll
          for (int j = 0; j < SK_PD; ++j) sk_issue(cur, j, true, wave, buf[j]);
        } else if (!sk_attention_idle(S)) {
          return;
        }
      }
      const SegDesc nxt = seg_desc(P, s + 1, nk, kept, share, share_o);
      // (a workgroup without attention work waits for the attention of the others: see sk_prefetch; every wave of an
      // attention workgroup is awaited at that workgroup's own barriers, so those do not linger)
      if (cur.kind == SEG_O && !attn_wg) sk_prefetch(nxt, SK_PF_ROUNDS, wave);
      if (cur.kind == SEG_O && cur.nrows > 0) {    // this wave's share of the attention output
        const bool ok = sk_stage_plain_slice(S.xs, p.attn + (size_t)b * nq, nq, tag_a, P.err, wave);
        if (lane == 0 && !ok) S.flag[12 + (s & 1)] = 0;
      }
      if (cur.gain != nullptr && D <= 4096) {      // this wave's share of the phase's normed input (sk_stage_norm_slice)
        float ssq = 0.f;
        const bool ok = sk_stage_norm_slice(S.xs, h, D, S.gs, tag_h, P.err, wave, ssq);
        if (lane == 0) { S.red[wave] = ssq; if (!ok) S.flag[12 + (s & 1)] = 0; }
      }
      lds_barrier();                               // input vector staged
      if (uni(*S.flag) == 0 || uni(S.flag[12 + (s & 1)]) == 0) return;
      // all blocks but the last request ahead inside this segment; the last one requests the first rounds of the
      // next segment (no per-round choice between the two descriptors)
      const int last0 = cur.nr_pad - SK_PD;
      const int* staged = cur.kind == SEG_DN ? S.flag + 2 : nullptr;
      const bool ahead = !(nxt.kind == SEG_O && attn_wg && wave < A.nact);     // a wave with tiles requests its output-projection rows afterwards
      int seen = 1;
      const bool progress = cur.kind == SEG_GU && cur.blk_stride != 0;     // the service wave sends z out block by block
      for (int r0 = 0; r0 < last0; r0 += SK_PD) {
#pragma unroll
        for (int j = 0; j < SK_PD; ++j) {
          sk_consume(cur, r0 + j, wave, buf[j], xsrc, S.psum, staged, seen);
          if (progress && lane == 0) __hip_atomic_store(S.flag + 4 + wave, r0 + j + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
          sk_issue(cur, r0 + j + SK_PD, true, wave, buf[j]);
        }
      }
#pragma unroll
      for (int j = 0; j < SK_PD; ++j) {
        sk_consume(cur, last0 + j, wave, buf[j], xsrc, S.psum, staged, seen);
        if (progress && lane == 0) __hip_atomic_store(S.flag + 4 + wave, last0 + j + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        sk_issue(nxt, j, ahead, wave, buf[j]);
      }
      lds_barrier();                               // partial sums complete
      if (cur.kind == SEG_O || cur.kind == SEG_DN) tag_h ^= 1u;     // (the service wave is writing h with the other tag now)
      cur = nxt;
    }
  }
#undef SK_STAMP
}

}  // namespace first
