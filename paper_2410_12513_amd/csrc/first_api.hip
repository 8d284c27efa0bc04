// C ABI of the router-gated prefill/decode library (see include/first.h).
// Host runtime: context, paged KV allocator, mask store, kept-index compaction, graph cache.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/first.h"
#include "decode_kernels.h"
#include "prefill_kernels.h"
#include "step_kernel.h"
#include "decode_batch_kernels.h"
#include "sample_kernels.h"
#include "train_kernels.h"

using namespace first;

// Scratch of first_sample_top_k_static, the entry point that allocates nothing: the per-chunk candidate lists of
// its first stage.  Every device the library runs on holds its own copy of the array (at its own address) until
// the process ends.  Host code never uses the array's name as an address: g_scratch_ptr[device] is what
// hipGetSymbolAddress returned with that device current.
constexpr long long STATIC_SCRATCH_CANDS = 131072;           // 1 MiB of {logit, index} pairs
constexpr int STATIC_SCRATCH_MAX_DEV = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_CANDS * 8];
static void* g_scratch_ptr[STATIC_SCRATCH_MAX_DEV] = {};
static std::mutex g_scratch_mutex;

namespace {

thread_local std::string g_create_error;


struct LayerPtrs {
  const void *wq, *wk, *wv, *wo, *wg, *wu, *wd;
  const float *g_attn, *g_mlp;
  bf16 *t_qkv = nullptr, *t_o = nullptr, *t_g = nullptr, *t_u = nullptr, *t_d = nullptr;   // tile-order copies (batched decode)
  bf16* wd_perm = nullptr;     // persistent kernel: down-projection matrix with its columns in z' order (sk_zperm_source)
};

}  // namespace

struct first_ctx {
  first_model_desc d{};
  hipStream_t stream = nullptr;
  bool own_stream = false;
  int num_cu = 256;
  std::string err;
  // weights (borrowed)
  const void* embed = nullptr;
  const void* lm_head = nullptr;
  const float* g_final = nullptr;
  const float* router = nullptr;
  std::vector<LayerPtrs> layers;
  // derived geometry
  int nq = 0, nkv = 0, half = 0, G = 1, max_pages = 0, n_pages = 0;
  size_t elem = 2, page_elems = 0;
  // device state
  std::vector<void*> allocs;
  char* kv_pool = nullptr;
  int *d_page_table = nullptr, *d_len = nullptr, *d_kept = nullptr, *d_nkept = nullptr;
  uint8_t* d_mask = nullptr;
  float* d_rho = nullptr;
  double* d_theta = nullptr;
  float *d_h = nullptr, *d_qkv = nullptr, *d_attn = nullptr, *d_z = nullptr, *d_part_o = nullptr, *d_part_ml = nullptr;
  unsigned *d_attn_cnt = nullptr, *d_head_cnt = nullptr;
  float* d_bg_part = nullptr;             // k_bgemv_g: [workgroups][16 slots][128 rows] partial sums of the K-slices
  unsigned* d_bg_cnt = nullptr;           //            arrival counters per tile group (zero between launches)
  size_t bg_part_floats = 0, bg_cnt_n = 0;
  Cand* d_topk_part = nullptr;            // [max_batch][chunks][SMP_KMAX] per-chunk candidates of first_sample_top_k
  float* d_logits_own = nullptr;          // [max_batch][V] logits of a sampled step whose caller wants none
  Cand* d_step_cands = nullptr;           // [workgroups][SMP_KMAX] per-workgroup candidates of a sampled step of the persistent kernel
  float2* d_rope_cs = nullptr;
  Best* d_arg_part = nullptr;
  // prefill workspace
  float *p_H = nullptr, *p_q = nullptr, *p_k = nullptr, *p_v = nullptr, *p_g = nullptr, *p_u = nullptr, *p_sig = nullptr;
  void *p_x = nullptr, *p_a = nullptr, *p_z = nullptr;
  bf16 *p_qh = nullptr, *p_ql = nullptr, *p_kc = nullptr, *p_vt = nullptr;   // matrix-core prefill attention operands
  bf16 *p_xh = nullptr, *p_xl = nullptr, *p_ah = nullptr, *p_al = nullptr, *p_zh = nullptr, *p_zl = nullptr;   // split activations (bf16 models)
  int p_tp = 0;                           // key pitch of p_vt / rows of p_kc (max_seq_len padded to the key tile)
  int prefill_flash = 1;                  // FIRST_OPT_PREFILL_ATTN
  float2* p_cs = nullptr;
  // soft-skip forward (first_soft_forward; allocated at its first call)
  float *p_Hs = nullptr, *p_lg = nullptr, *p_ce = nullptr;
  // host state
  int B = 0;
  std::vector<int> hlen;
  std::vector<char> decoded;
  std::vector<std::vector<uint8_t>> hmask;
  std::vector<int> free_pages, page_order, h_page_table;
  std::vector<int> seq_npages;
  // layer slices of the KV pool: layer i's pages live in slice layer_slice[i].  Without elision slice = layer.
  // With elision (kv_layer_slots < n_layers) a layer gets a slice when the first sequence's router keeps it;
  // the prompt pass of a layer nobody keeps uses the one scratch slice behind the slots.
  bool kv_elide = false;
  int kv_slots = 0, slices_used = 0;
  std::vector<int> layer_slice;
  std::vector<std::vector<uint8_t>> has_kv;   // [seq][layer]: the sequence's prompt KV of that layer was stored
  uint8_t* h_keep = nullptr;                  // pinned: one router decision read back per layer while eliding
  hipEvent_t ev_keep = nullptr;
  // persistent whole-step kernel (bf16, one live sequence)
  LayerDev* d_layers = nullptr;
  unsigned* d_done = nullptr;             // [num_cu] per-workgroup epochs of the final reduction
  // batched decode (several live sequences): split activations, 1/rms per slot, logits when the caller wants none
  bf16 *d_xh = nullptr, *d_xl = nullptr, *d_zh = nullptr, *d_zl = nullptr, *d_x2h = nullptr, *d_x2l = nullptr;
  float* d_ssq = nullptr;                 // [SSQ_GROUPS][16] per-tile-group sums of squares (fused split of the O / down epilogues)
  float *d_rinv = nullptr, *d_logits_all = nullptr;
  int xpitch = 0;
  int batch_path = -1;                    // FIRST_OPT_BATCH_PATH
  bf16* t_head = nullptr;                 // tile-order copy of the LM head
  bool tiled = false;                     // tile-order copies of all matrices exist
  float *x_h = nullptr, *x_qkv = nullptr, *x_attn = nullptr, *x_z = nullptr;   // tagged exchange vectors (written by k_step only)
  float* x_part = nullptr;                // tagged partial attention results of key splits 1.. (sk_part_index)
  int* d_tagstate = nullptr;              // [B][8] tags of their latest writes, epoch of the latest final reduction
  int* d_err = nullptr;
  unsigned long long* d_tdbg = nullptr;   // step-kernel timestamps (FIRST_OPT_STEP_TIMING)
  int step_timing = 0;
  bool step_ok = false;        // geometry fits the persistent kernel
  bool zperm = false;          // ... and every layer has its column-permuted copy of the down-projection matrix
  size_t step_lds = 0;
  // options and graph cache
  int use_graph = 1, attn_splits = 0, decode_path = -1;   // -1: persistent kernel when possible
  struct CachedGraph { hipGraphExec_t exec; unsigned long long used; };
  std::map<std::string, CachedGraph> graphs;
  unsigned long long graph_clock = 0;
};

namespace {

int fail(first_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_create_error = msg;
  return code;
}

#define HIPCHK(c, expr)                                                                      \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess)                                                                    \
      return fail((c), FIRST_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));    \
  } while (0)

template <typename T>
int dev_alloc(first_ctx* c, T** out, size_t count) {
  void* p = nullptr;
  HIPCHK(c, hipMalloc(&p, count * sizeof(T) + 256));
  c->allocs.push_back(p);
  *out = reinterpret_cast<T*>(p);
  return FIRST_OK;
}

int device_cus() {
  static int cus = 0;
  if (!cus) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      cus = prop.multiProcessorCount;
    if (cus <= 0) cus = 256;
  }
  return cus;
}

// workgroups for a mat-vec over `rows` rows with R rows per wave iteration
int gemv_grid(int rows, int R, int num_cu) {
  const int need = (rows + WAVES * R - 1) / (WAVES * R);
  return std::max(1, std::min(need, num_cu * 4));
}

// Tagged exchange of the persistent kernel: all-zero vectors and "latest tag 0" are a consistent start.
hipError_t reset_tagged_exchange(first_ctx* c) {
  const size_t Bm = (size_t)c->d.max_batch;
  hipError_t e = hipMemset(c->x_h, 0, Bm * c->d.d_model * sizeof(float));
  if (e == hipSuccess) e = hipMemset(c->x_qkv, 0, Bm * (c->nq + 2 * c->nkv) * sizeof(float));
  if (e == hipSuccess) e = hipMemset(c->x_attn, 0, Bm * c->nq * sizeof(float));
  if (e == hipSuccess) e = hipMemset(c->x_z, 0, Bm * c->d.d_ffn * sizeof(float));
  if (e == hipSuccess) e = hipMemset(c->x_part, 0, sk_part_index(c->d.n_q_heads, c->d.head_dim, (int)Bm, 0, 0) * sizeof(float));
  if (e == hipSuccess) e = hipMemset(c->d_tagstate, 0, Bm * 8 * sizeof(int));
  if (e == hipSuccess) e = hipMemset(c->d_done, 0, (size_t)c->num_cu * sizeof(unsigned));
  return e;
}

size_t kv_slice_bytes(const first_ctx* c) { return (size_t)c->n_pages * c->page_elems * c->elem; }

// Page pool of layer i: its slice, or the scratch slice when the layer has none (only while eliding).
char* kv_base(const first_ctx* c, int i) {
  const int s = c->layer_slice[i] >= 0 ? c->layer_slice[i] : c->kv_slots;
  return c->kv_pool + (size_t)s * kv_slice_bytes(c);
}

void reset_layer_slices(first_ctx* c) {
  const int L = c->d.n_layers;
  c->layer_slice.resize(L);
  for (int i = 0; i < L; ++i) c->layer_slice[i] = c->kv_elide ? -1 : i;
  c->slices_used = c->kv_elide ? 0 : L;
  for (auto& h : c->has_kv) std::fill(h.begin(), h.end(), 0);
}

void release_sequences(first_ctx* c) {
  c->B = 0;
  c->free_pages.assign(c->page_order.rbegin(), c->page_order.rend());   // pop_back hands out page_order[0] first
  std::fill(c->seq_npages.begin(), c->seq_npages.end(), 0);
  std::fill(c->decoded.begin(), c->decoded.end(), 0);
  reset_layer_slices(c);
}

// Column-permuted copies of the down-projection matrices for the persistent kernel's blocked gate/up phase (as much
// memory again as those matrices: 117 MB per layer on the 8B shape), made only when the geometry allows the blocks and
// at least that much device memory plus a 4 GiB margin is free; without them z keeps its natural order and the down
// projection waits for the end of the gate/up phase.  The caller's matrices must not change afterwards.
hipError_t make_permuted_down_copies(first_ctx* c) {
  const first_model_desc& d = c->d;
  if (!sk_zperm_fits(d.d_ffn, d.d_model, c->num_cu)) return hipSuccess;
  const size_t per_layer = (size_t)d.d_model * d.d_ffn * sizeof(bf16);
  size_t free_b = 0, total_b = 0;
  if (hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < per_layer * d.n_layers + ((size_t)4 << 30)) return hipSuccess;
  for (int i = 0; i < d.n_layers; ++i) {
    LayerPtrs& l = c->layers[i];
    if (dev_alloc(c, &l.wd_perm, (size_t)d.d_model * d.d_ffn)) return hipErrorOutOfMemory;
    hipLaunchKernelGGL(k_permute_down_columns, dim3(4096), dim3(WG), 0, c->stream, reinterpret_cast<const bf16*>(l.wd), l.wd_perm,
                       d.d_model, d.d_ffn, c->num_cu);
  }
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e == hipSuccess) e = hipGetLastError();
  c->zperm = e == hipSuccess;
  return e;
}

// Per-layer pointers of the persistent kernel (weights, gains, the layer's page pool).  The stream must be idle.
hipError_t upload_layer_table(first_ctx* c) {
  const int L = c->d.n_layers;
  std::vector<LayerDev> ld(L);
  for (int i = 0; i < L; ++i) {
    const LayerPtrs& l = c->layers[i];
    ld[i] = LayerDev{(const bf16*)l.wq, (const bf16*)l.wk, (const bf16*)l.wv, (const bf16*)l.wo, (const bf16*)l.wg,
                     (const bf16*)l.wu, c->zperm ? l.wd_perm : (const bf16*)l.wd, l.g_attn, l.g_mlp, (bf16*)kv_base(c, i)};
  }
  return hipMemcpy(c->d_layers, ld.data(), L * sizeof(LayerDev), hipMemcpyHostToDevice);
}

// (an executable graph may still be running on the stream: wait before destroying it)
void drop_graphs(first_ctx* c) {
  if (c->graphs.empty()) return;
  (void)hipStreamSynchronize(c->stream);
  for (auto& kv : c->graphs) (void)hipGraphExecDestroy(kv.second.exec);
  c->graphs.clear();
}

// A wait between workgroups of the persistent kernel that gave up says so in d_err; every later launch then leaves at
// its first wait.  Called by the entry points that have just synchronised the stream: reports it once and starts the
// exchange state afresh.
int check_step_error(first_ctx* c, const char* who) {
  int err = 0;
  HIPCHK(c, hipMemcpy(&err, c->d_err, sizeof(int), hipMemcpyDeviceToHost));
  if (err & 1) {                                   // (the bits above bit 0: a poll limit set by FIRST_OPT_STEP_POLL_LIMIT, gone with the error)
    (void)hipMemset(c->d_err, 0, 4 * sizeof(int));
    (void)reset_tagged_exchange(c);
    return fail(c, FIRST_ERR_HIP, std::string(who) + ": a wait between workgroups of the persistent decode kernel gave up; "
                                  "the tokens and logits of the steps since are not valid");
  }
  return FIRST_OK;
}

DecParams base_params(const first_ctx* c, int b, int S) {
  DecParams p{};
  const first_model_desc& d = c->d;
  p.D = d.d_model; p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.hd = d.head_dim; p.F = d.d_ffn; p.V = d.vocab;
  p.G = c->G; p.P = d.kv_page_tokens; p.max_pages = c->max_pages; p.S = S;
  p.eps = d.rms_eps; p.qscale = 1.0f / std::sqrt((float)d.head_dim);
  p.b = b;
  p.h = c->d_h; p.qkv = c->d_qkv; p.attn = c->d_attn; p.z = c->d_z;
  p.part_o = c->d_part_o; p.part_ml = c->d_part_ml; p.attn_cnt = c->d_attn_cnt;
  p.rope_cs = c->d_rope_cs; p.len = c->d_len; p.page_table = c->d_page_table; p.theta = c->d_theta;
  p.embed = c->embed; p.lm_head = c->lm_head; p.g_final = c->g_final;
  p.arg_part = c->d_arg_part; p.head_cnt = c->d_head_cnt;
  p.page_elems = c->page_elems;
  return p;
}

void set_layer(const first_ctx* c, DecParams& p, int i) {
  const LayerPtrs& l = c->layers[i];
  p.wq = l.wq; p.wk = l.wk; p.wv = l.wv; p.wo = l.wo; p.wg = l.wg; p.wu = l.wu; p.wd = l.wd;
  p.g_attn = l.g_attn; p.g_mlp = l.g_mlp;
  p.kv_layer = kv_base(c, i);
}

template <typename WT>
size_t attn_lds(const first_ctx* c) {
  const size_t kpitch = (size_t)c->d.head_dim * sizeof(WT) + 4;
  return ((size_t)c->G * c->d.head_dim + 2 * c->d.head_dim + 4) * sizeof(float) + 64 * kpitch +
         64 * (size_t)c->d.head_dim * sizeof(WT);
}

// LM head of sequence p.b (also used for the first token after prefill); logits / token_out
// are the [B, ...] base pointers.
template <typename WT>
void enqueue_head(first_ctx* c, DecParams p, float* logits, int* token_out, int advance) {
  p.logits = logits; p.token_out = token_out; p.advance_len = advance;
  const int grid = std::min(gemv_grid(c->d.vocab, 4, c->num_cu), ARG_MAX_WG);
  const size_t lds = ((size_t)c->d.d_model + WAVES) * sizeof(float) + WAVES * sizeof(Best) + 16;
  hipLaunchKernelGGL(k_head<WT>, dim3(grid), dim3(WG), lds, c->stream, p);
}

// One decode token for every live sequence, one kernel per fused op, kept layers only.
template <typename WT>
void enqueue_decode_ops(first_ctx* c, const int* tokens, float* logits, int* token_out, int S) {
  const first_model_desc& d = c->d;
  const size_t lds_d = ((size_t)d.d_model + WAVES) * sizeof(float);
  const size_t lds_o = ((size_t)c->nq + WAVES) * sizeof(float);
  const size_t lds_f = ((size_t)d.d_ffn + WAVES) * sizeof(float);
  const int g_qkv = gemv_grid(c->nq + 2 * c->nkv, 4, c->num_cu);
  const int g_o = gemv_grid(d.d_model, 4, c->num_cu);
  const int g_gu = gemv_grid(2 * d.d_ffn, 4, c->num_cu);
  for (int b = 0; b < c->B; ++b) {
    DecParams p = base_params(c, b, S);
    p.tokens = tokens;
    hipLaunchKernelGGL(k_embed<WT>, dim3(1), dim3(WG), 0, c->stream, p);
    for (int i = 0; i < d.n_layers; ++i) {
      if (!c->hmask[b][i]) continue;            // skipped layer: no launch, no bytes
      set_layer(c, p, i);
      hipLaunchKernelGGL(k_qkv<WT>, dim3(g_qkv), dim3(WG), lds_d, c->stream, p);
      hipLaunchKernelGGL(k_attn<WT>, dim3(S, d.n_kv_heads), dim3(WG), attn_lds<WT>(c), c->stream, p);
      hipLaunchKernelGGL(k_oproj<WT>, dim3(g_o), dim3(WG), lds_o, c->stream, p);
      hipLaunchKernelGGL(k_gateup<WT>, dim3(g_gu), dim3(WG), lds_d, c->stream, p);
      hipLaunchKernelGGL(k_down<WT>, dim3(g_o), dim3(WG), lds_f, c->stream, p);
    }
    enqueue_head<WT>(c, p, logits, token_out, 1);
  }
}

// Shape of a batched mat-vec over N rows: RT row tiles per wave (they share the activation
// operands), K-slices over the 8 waves of a workgroup when N alone does not fill the chip.
template <int MODE, int RT>
void launch_bgemv_rt(first_ctx* c, const BatchParams& P, int N, int K) {
  const bool tiled = c->tiled;
  const int groups = ((N + 15) / 16 + RT - 1) / RT;
  int ks = 1;
  while (ks < BG_WAVES && groups * ks < 6 * c->num_cu) ks *= 2;       // (6 waves per CU measured best of 3 / 6 / 12 / 24)
  const int groups_per_wg = BG_WAVES / ks;
  const int grid = (groups + groups_per_wg - 1) / groups_per_wg;
  if (tiled) hipLaunchKernelGGL((k_bgemv<MODE, RT, true>), dim3(grid), dim3(BG_THREADS), 0, c->stream, P, N, K, ks);
  else hipLaunchKernelGGL((k_bgemv<MODE, RT, false>), dim3(grid), dim3(BG_THREADS), 0, c->stream, P, N, K, ks);
}

bool d_batch_fits(const first_ctx* c) {
  return c->d.d_model % 8 == 0 && c->nq % 8 == 0 && c->d.d_ffn % 8 == 0;
}

// Mat-vecs with tile-order weights as (GW row tiles) x (one slice of K) per workgroup (k_bgemv_g): GW in
// 5..8 and at most 8 slices, chosen so that the workgroups fill whole rounds over the compute units
// (ties: more waves per workgroup, fewer slices).
template <int MODE, int GW>
void launch_bgemv_gw(first_ctx* c, const BatchParams& P, int N, int K, int groups, int ks) {
  hipLaunchKernelGGL((k_bgemv_g<MODE, GW>), dim3(groups * ks), dim3(GW * 64), (size_t)2 * bgg_per(K, ks) * 1024, c->stream, P, N, K, ks,
                     c->d_bg_part, c->d_bg_cnt);
}

// Returns the number of tile groups launched (0: this decomposition is not available, nothing was launched).
template <int MODE>
int launch_bgemv_g(first_ctx* c, const BatchParams& P, int N, int K) {
  if (!c->tiled || c->d_bg_part == nullptr) return 0;
  constexpr int NS = MODE == BG_GU ? 2 : 1;
  const int tiles = (N + 15) / 16, ksteps = (K + 31) / 32;
  int best_gw = 0, best_ks = 0;
  double best = 0.0;
  for (int gw = 8; gw >= 5; --gw)
    for (int ks = 1; ks <= std::min(8, ksteps); ++ks) {
      const int groups = (tiles + gw - 1) / gw, wgs = groups * ks;
      if ((size_t)2 * bgg_per(K, ks) * 1024 > 150 * 1024) continue;
      if ((size_t)wgs * NS * 16 * gw * 16 > c->bg_part_floats || (size_t)groups > c->bg_cnt_n) continue;
      // useful wave-slots over the wave-slots of the rounds the grid occupies
      const int rounds = (wgs + c->num_cu - 1) / c->num_cu;
      const double eff = (double)tiles * ks / ((double)rounds * c->num_cu * gw) / rounds;
      if (eff > best + 1e-9) { best = eff; best_gw = gw; best_ks = ks; }
    }
  if (best_gw == 0) return 0;
  const int groups = (tiles + best_gw - 1) / best_gw;
  switch (best_gw) {
    case 8: launch_bgemv_gw<MODE, 8>(c, P, N, K, groups, best_ks); break;
    case 7: launch_bgemv_gw<MODE, 7>(c, P, N, K, groups, best_ks); break;
    case 6: launch_bgemv_gw<MODE, 6>(c, P, N, K, groups, best_ks); break;
    default: launch_bgemv_gw<MODE, 5>(c, P, N, K, groups, best_ks); break;
  }
  return groups;
}

// Returns the number of tile groups whose epilogues honoured P.fuse_gain (0: the kernel used does not fuse).
template <int MODE>
int launch_bgemv(first_ctx* c, const BatchParams& P, int N, int K) {
  if constexpr (MODE == BG_QKV || MODE == BG_O || MODE == BG_DN || MODE == BG_GU) {
    const int groups = launch_bgemv_g<MODE>(c, P, N, K);
    if (groups) return groups;
  }
  // two tiles per wave once that still leaves every SIMD several waves
  if ((N + 15) / 16 >= 16 * c->num_cu / 8) launch_bgemv_rt<MODE, 2>(c, P, N, K);
  else launch_bgemv_rt<MODE, 1>(c, P, N, K);
  return 0;
}

// Tile-order copies of every matrix for the batched mat-vecs (as much again as the weights),
// made only when at least that much device memory plus a 4 GiB margin is free; without them
// the batched path reads the caller's row-major matrices.
hipError_t make_tiled_copies(first_ctx* c) {
  const first_model_desc& d = c->d;
  auto tiled_elems = [](int N, int K) { return (size_t)((N + 15) / 16) * ((K + 31) / 32) * 512; };
  const int nqkv = c->nq + 2 * c->nkv;
  const size_t per_layer = tiled_elems(nqkv, d.d_model) + tiled_elems(d.d_model, c->nq) + 2 * tiled_elems(d.d_ffn, d.d_model) +
                           tiled_elems(d.d_model, d.d_ffn);
  const size_t total = (per_layer * d.n_layers + tiled_elems(d.vocab, d.d_model)) * sizeof(bf16);
  size_t free_b = 0, total_b = 0;
  if (hipMemGetInfo(&free_b, &total_b) != hipSuccess || free_b < total + ((size_t)4 << 30)) return hipSuccess;
  auto conv = [&](const void* src, bf16* dst, int N, int K) {
    const size_t items = tiled_elems(N, K) / 8;
    hipLaunchKernelGGL(k_tile_weights, dim3((unsigned)std::min<size_t>((items + WG - 1) / WG, 65535)), dim3(WG), 0, c->stream,
                       reinterpret_cast<const bf16*>(src), dst, N, K);
  };
  for (int i = 0; i < d.n_layers; ++i) {
    LayerPtrs& l = c->layers[i];
    if (dev_alloc(c, &l.t_qkv, tiled_elems(nqkv, d.d_model)) || dev_alloc(c, &l.t_o, tiled_elems(d.d_model, c->nq)) ||
        dev_alloc(c, &l.t_g, tiled_elems(d.d_ffn, d.d_model)) || dev_alloc(c, &l.t_u, tiled_elems(d.d_ffn, d.d_model)) ||
        dev_alloc(c, &l.t_d, tiled_elems(d.d_model, d.d_ffn)))
      return hipErrorOutOfMemory;
    // q, k and v stacked: nq and nkv are multiples of 64, so no tile straddles two matrices
    conv(l.wq, l.t_qkv, c->nq, d.d_model);
    conv(l.wk, l.t_qkv + tiled_elems(c->nq, d.d_model), c->nkv, d.d_model);
    conv(l.wv, l.t_qkv + tiled_elems(c->nq + c->nkv, d.d_model), c->nkv, d.d_model);
    conv(l.wo, l.t_o, d.d_model, c->nq);
    conv(l.wg, l.t_g, d.d_ffn, d.d_model);
    conv(l.wu, l.t_u, d.d_ffn, d.d_model);
    conv(l.wd, l.t_d, d.d_model, d.d_ffn);
  }
  if (dev_alloc(c, &c->t_head, tiled_elems(d.vocab, d.d_model))) return hipErrorOutOfMemory;
  conv(c->lm_head, c->t_head, d.vocab, d.d_model);
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e == hipSuccess) e = hipGetLastError();
  c->tiled = e == hipSuccess;
  return e;
}

// One decode token for every live sequence (bf16 models), layer by layer: the sequences that
// keep a layer go through it together, so its weights are read once per step and per group
// of BATCH_SLOTS sequences whatever the masks are.
void enqueue_decode_batched(first_ctx* c, const int* tokens, float* logits, int* token_out, int S) {
  const first_model_desc& d = c->d;
  const int nqkv = c->nq + 2 * c->nkv;
  // attention on register-resident key tiles when the geometry allows, one 64-key tile per
  // worker wave group and split where the longest sequence permits
  const bool tiles_attn = (d.head_dim == 64 || d.head_dim == 128) && c->G <= SK_WAVES && d.kv_page_tokens == 16;
  const int nkg = std::max(1, SK_WAVES / c->G);
  const int nsplit = std::max(1, std::min(S_MAX, (2 * S + nkg - 1) / nkg));
  const size_t attn_tiles_lds = sk_lds_floats(0, 0, 0, c->G, d.head_dim) * sizeof(float);
  // models with 4 query heads per KV head and head dimension 128: tiles fetched once per workgroup, scores on the matrix cores
  const bool shared_attn = c->G == 4 && d.head_dim == 128;
  for (int b0 = 0; b0 < c->B; b0 += BATCH_SLOTS) {
    BatchParams P{};
    P.d = base_params(c, 0, S);
    P.d.tokens = tokens; P.d.token_out = token_out;
    P.xh = c->d_xh; P.xl = c->d_xl; P.zh = c->d_zh; P.zl = c->d_zl; P.rinv = c->d_rinv; P.xpitch = c->xpitch;
    P.x2h = c->d_x2h; P.x2l = c->d_x2l; P.ssq_part = c->d_ssq; P.fuse_gain = nullptr; P.ssq_groups = 0;
    P.logits_all = logits ? logits : c->d_logits_all;
    P.t_head = c->t_head;
    SeqList all{};
    for (int b = b0; b < std::min(c->B, b0 + BATCH_SLOTS); ++b) all.id[all.n++] = b;
    P.seqs = all;
    hipLaunchKernelGGL(k_embed_b, dim3(all.n), dim3(WG), 0, c->stream, P);
    auto xsplit = [&](int src, int K, const float* gain) {
      const int chunk = 1024;
      hipLaunchKernelGGL(k_xsplit, dim3(P.seqs.n, (K + chunk - 1) / chunk), dim3(WG), 0, c->stream, P, src, K, chunk, gain);
    };
    // slot lists per layer (a layer nobody keeps has none); the list after the last layer is everybody (final norm)
    std::vector<SeqList> keeps(d.n_layers + 1);
    for (int i = 0; i < d.n_layers; ++i)
      for (int j = 0; j < all.n; ++j)
        if (c->hmask[all.id[j]][i]) keeps[i].id[keeps[i].n++] = all.id[j];
    keeps[d.n_layers] = all;
    auto same_list = [](const SeqList& a, const SeqList& b) {
      if (a.n != b.n) return false;
      for (int j = 0; j < a.n; ++j)
        if (a.id[j] != b.id[j]) return false;
      return true;
    };
    // x_groups > 0: xh / xl already hold the split input of the coming norm op for its slot list, left there by the
    // previous down projection's epilogue together with that many partial sums of squares
    int x_groups = 0;
    for (int i = 0; i < d.n_layers; ++i) {
      const SeqList& keep = keeps[i];
      if (keep.n == 0) continue;                   // skipped by every sequence: no launch, no bytes
      P.seqs = keep;
      set_layer(c, P.d, i);
      { const LayerPtrs& l = c->layers[i]; P.t_qkv = l.t_qkv; P.t_o = l.t_o; P.t_g = l.t_g; P.t_u = l.t_u; P.t_d = l.t_d; }
      if (x_groups == 0) xsplit(0, d.d_model, P.d.g_attn);
      P.ssq_groups = x_groups;
      launch_bgemv<BG_QKV>(c, P, nqkv, d.d_model);
      P.ssq_groups = 0;
      // shared key / value tiles: about one workgroup per compute unit, long loops
      int ns_shared = std::max(1, std::min(S_MAX, c->num_cu / std::max(1, d.n_kv_heads * keep.n)));
      if (c->attn_splits > 0) ns_shared = std::min(ns_shared, c->attn_splits);
      // a split's page ids must fit the kernel's LDS table whatever length a sequence reaches (a bound that
      // does not move with the lengths, so a captured graph stays valid)
      ns_shared = std::max(ns_shared, ((d.max_seq_len + 64) / 64 * 4 + AS_PT - 1) / AS_PT);
      P.attn_nwork = 0;
      if (tiles_attn && shared_attn && c->attn_splits <= 0) {
        // work list: splits in proportion to each sequence's length - the fewest tiles per workgroup for which the batch
        // still fits one round of the compute units at today's lengths (a cached graph keeps the list while the
        // sequences grow: their splits just get longer)
        const int min_sp = ((d.max_seq_len + 64) / 64 * 4 + AS_PT - 1) / AS_PT;    // a split's page ids fit the LDS table
        int sp[BATCH_SLOTS];
        for (int tpw = AS_NT; tpw <= AS_PT / 4; ++tpw) {
          int wgs = 0;
          for (int j = 0; j < keep.n; ++j) {
            sp[j] = std::min(S_MAX, std::max(min_sp, (c->hlen[keep.id[j]] / 64 + 1 + tpw - 1) / tpw));
            wgs += sp[j];
          }
          if (wgs * d.n_kv_heads <= c->num_cu || tpw == AS_PT / 4) {
            if (wgs <= ATTN_WORK_MAX)
              for (int j = 0; j < keep.n; ++j)
                for (int q = 0; q < sp[j]; ++q)
                  P.attn_work[P.attn_nwork++] = attn_work_pack(j, q, sp[j]);
            break;
          }
        }
      }
      if (tiles_attn && shared_attn && P.attn_nwork > 0)
        hipLaunchKernelGGL((k_attn_mfma_b<128, 4>), dim3(d.n_kv_heads, P.attn_nwork), dim3(AS_THREADS), as_lds_bytes(4, 128), c->stream, P);
      else if (tiles_attn && shared_attn)
        hipLaunchKernelGGL((k_attn_mfma_b<128, 4>), dim3(ns_shared, d.n_kv_heads, keep.n), dim3(AS_THREADS), as_lds_bytes(4, 128), c->stream, P);
      else if (tiles_attn && d.head_dim == 128)
        hipLaunchKernelGGL(k_attn_tiles_b<128>, dim3(nsplit, d.n_kv_heads, keep.n), dim3(AT_THREADS), attn_tiles_lds, c->stream, P);
      else if (tiles_attn)
        hipLaunchKernelGGL(k_attn_tiles_b<64>, dim3(nsplit, d.n_kv_heads, keep.n), dim3(AT_THREADS), attn_tiles_lds, c->stream, P);
      else
        hipLaunchKernelGGL(k_attn_b, dim3(S, d.n_kv_heads, keep.n), dim3(WG), attn_lds<bf16>(c), c->stream, P);
      if (!tiles_attn) xsplit(1, c->nq, nullptr);        // (the tile kernels write their output already split)
      // output projection; its epilogue leaves the MLP norm's input behind when it can
      P.fuse_gain = P.d.g_mlp;
      int groups = launch_bgemv<BG_O>(c, P, d.d_model, c->nq);
      P.fuse_gain = nullptr;
      if (groups == 0) xsplit(0, d.d_model, P.d.g_mlp);
      P.ssq_groups = groups;
      launch_bgemv<BG_GU>(c, P, d.d_ffn, d.d_model);
      P.ssq_groups = 0;
      // down projection; the next norm op (the next layer somebody keeps, or the final norm) can take its input
      // from the epilogue if it runs on the same slot list
      int nx = i + 1;
      while (nx < d.n_layers && keeps[nx].n == 0) ++nx;
      P.fuse_gain = nx < d.n_layers ? c->layers[nx].g_attn : c->g_final;
      if (!same_list(keeps[nx], keep)) P.next = keeps[nx];      // (the epilogue then writes the consumer's slots)
      groups = launch_bgemv<BG_DN>(c, P, d.d_model, d.d_ffn);
      P.fuse_gain = nullptr; P.next.n = 0;
      x_groups = groups;
    }
    P.seqs = all;
    if (x_groups == 0) xsplit(0, d.d_model, c->g_final);
    P.ssq_groups = x_groups;
    launch_bgemv<BG_HEAD>(c, P, d.vocab, d.d_model);
    P.ssq_groups = 0;
    hipLaunchKernelGGL(k_argmax_part_b, dim3(all.n, ARG_CHUNKS), dim3(WG), 0, c->stream, P);
    hipLaunchKernelGGL(k_argmax_final_b, dim3(all.n), dim3(64), 0, c->stream, P, 1);
  }
}

// The instantiation of the persistent kernel for this context's head dimension.
const void* step_kernel_fn(const first_ctx* c) {
  return c->d.head_dim == 128 ? reinterpret_cast<const void*>(&k_step<128>) : reinterpret_cast<const void*>(&k_step<64>);
}

// What a sampled step adds to a greedy one (null: greedy).
struct SampleArgs { const float* uniforms; float temperature; int top_k; int* candidates_out; };

// One decode token of the single live sequence as one persistent kernel.

void enqueue_decode_step_kernel(first_ctx* c, const int* tokens, float* logits, int* token_out, const SampleArgs* smp = nullptr) {
  StepParams P{};
  P.d = base_params(c, 0, 1);
  P.d.tokens = tokens; P.d.logits = logits; P.d.token_out = token_out; P.d.advance_len = 1;
  P.layers = c->d_layers; P.kept = c->d_kept; P.n_kept = c->d_nkept; P.L = c->d.n_layers;
  P.done = c->d_done; P.err = c->d_err;
  P.tagstate = c->d_tagstate; P.h_out = c->d_h; P.part = c->x_part; P.zperm = c->zperm ? 1 : 0;
  P.d.h = c->x_h; P.d.qkv = c->x_qkv; P.d.attn = c->x_attn; P.d.z = c->x_z;
  P.tdbg = c->step_timing ? c->d_tdbg : nullptr;
  if (smp) {
    P.smp_k = smp->top_k; P.smp_temperature = smp->temperature; P.smp_u = smp->uniforms;
    P.smp_part = c->d_step_cands; P.smp_cand_out = smp->candidates_out;
  }
  hipLaunchKernelGGL(reinterpret_cast<void (*)(StepParams)>(const_cast<void*>(step_kernel_fn(c))), dim3(c->num_cu), dim3(SK_THREADS),
                     c->step_lds, c->stream, P);
}

// Does the geometry fit the persistent kernel's static work split?
bool step_kernel_fits(const first_ctx* c) {
  const first_model_desc& d = c->d;
  if (d.dtype != FIRST_DTYPE_BF16) return false;
  if (d.d_model % 256 || c->nq % 256 || d.d_ffn % 256) return false;           // row segments may be partial, rows stay 512-byte aligned
  if (c->G > SK_SWAVES || d.kv_page_tokens != 16) return false;               // one streaming wave per query head of a KV group
  const int ncu = c->num_cu;
  if (d.n_q_heads > ncu || d.d_ffn > 16384 || d.d_model > 64 * ncu || d.d_model > 16384 || c->nq > 16384) return false;   // (one residual row per service-wave lane)
  if ((long long)std::max({d.vocab, 2 * d.d_ffn, c->nq + 2 * c->nkv}) * (ncu + 1) >= (1LL << 31)) return false;
  // (one residual row per service-wave lane: at most 64 rows of the output / down projection per workgroup)
  auto units = [&](long long rows, int K) { return (int)((rows + ncu - 1) / ncu + 2) * ((K + SK_SEG - 1) / SK_SEG); };
  const int worst = std::max({units(d.vocab, d.d_model), units(c->nq + 2 * c->nkv, d.d_model), 66 * ((c->nq + SK_SEG - 1) / SK_SEG),
                              units(2LL * d.d_ffn, d.d_model), units(d.d_model, d.d_ffn)});
  if (worst > SK_PSUM) return false;
  return sk_lds_floats(d.d_model, c->nq, d.d_ffn, c->G, d.head_dim) * sizeof(float) <= 150 * 1024;
}

// a_fp32: the activations are fp32 (prefill path); bf16 weights then use the split-precision
// matrix-core kernel.
int launch_gemm(first_ctx* c, hipStream_t st, int dtype, const void* A, const void* W, float* C, int M, int N,
                int K, int acc, bool a_fp32 = false) {
  if (dtype == FIRST_DTYPE_BF16 && a_fp32) {
    dim3 grid((N + GB_N - 1) / GB_N, (M + GB_M - 1) / GB_M);
    hipLaunchKernelGGL(k_gemm_nt_bf16_split, grid, dim3(WG), 0, st, reinterpret_cast<const float*>(A),
                       reinterpret_cast<const bf16*>(W), C, M, N, K, acc);
  } else if (dtype == FIRST_DTYPE_BF16) {
    dim3 grid((N + GB_N - 1) / GB_N, (M + GB_M - 1) / GB_M);
    hipLaunchKernelGGL(k_gemm_nt_bf16, grid, dim3(WG), 0, st, reinterpret_cast<const bf16*>(A),
                       reinterpret_cast<const bf16*>(W), C, M, N, K, acc);
  } else {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    hipLaunchKernelGGL(k_gemm_nt_f32, grid, dim3(WG), 0, st, reinterpret_cast<const float*>(A),
                       reinterpret_cast<const float*>(W), C, M, N, K, acc);
  }
  HIPCHK(c, hipGetLastError());
  return FIRST_OK;
}

int launch_gemm_hl(first_ctx* c, hipStream_t st, const bf16* Ah, const bf16* Al, const void* W, float* C, int M, int N, int K,
                   int acc) {
  dim3 grid((N + GB_N - 1) / GB_N, (M + GB_M - 1) / GB_M);
  if (M > GB_MS && (int)(grid.x * grid.y) <= device_cus()) {   // at most one 128-row tile per compute unit: use 64-row tiles
    dim3 gs(grid.x, (M + GB_MS - 1) / GB_MS);
    hipLaunchKernelGGL(k_gemm_nt_bf16_hl_s, gs, dim3(WG), 0, st, Ah, Al, reinterpret_cast<const bf16*>(W), C, M, N, K, acc);
    HIPCHK(c, hipGetLastError());
    return FIRST_OK;
  }
  hipLaunchKernelGGL(k_gemm_nt_bf16_hl, grid, dim3(WG), 0, st, Ah, Al, reinterpret_cast<const bf16*>(W), C, M, N, K, acc);
  HIPCHK(c, hipGetLastError());
  return FIRST_OK;
}

// Up to three projections of the same split activations in one launch.
int launch_gemm_hl_seg(first_ctx* c, hipStream_t st, const bf16* Ah, const bf16* Al, int M, int K, int acc,
                       std::initializer_list<GemmSeg> list) {
  GemmSegs segs{};
  int blocks = 0;
  for (const GemmSeg& g : list) {
    GemmSeg s = g;
    s.blocks = (g.N + GB_N - 1) / GB_N;
    blocks += s.blocks;
    segs.s[segs.n++] = s;
  }
  hipLaunchKernelGGL(k_gemm_nt_bf16_hl_seg, dim3(blocks, (M + GB_M - 1) / GB_M), dim3(WG), 0, st, Ah, Al, segs, M, K, acc);
  HIPCHK(c, hipGetLastError());
  return FIRST_OK;
}

// Prompt attention on the matrix cores: operand preparation (query split, key gather, value
// transpose out of the cache pages) and the tiled kernel.
void launch_attn_flash(first_ctx* c, hipStream_t st, const bf16* pool, const int* pt, int T) {
  const first_model_desc& d = c->d;
  const size_t nq_all = (size_t)T * c->nq;
  hipLaunchKernelGGL(k_split_bf16, dim3((unsigned)std::min<size_t>((nq_all + WG - 1) / WG, 16384)), dim3(WG), 0, st, c->p_q,
                     c->p_qh, c->p_ql, nq_all);
  hipLaunchKernelGGL(k_kv_gather, dim3((T + 31) / 32, d.n_kv_heads), dim3(WG), 0, st, pool, c->page_elems, pt, c->p_kc,
                     c->p_vt, T, c->p_tp, d.n_kv_heads, d.head_dim, d.kv_page_tokens);
  const dim3 grid((T + WAVES * FA_QW - 1) / (WAVES * FA_QW), d.n_q_heads);
  if (d.head_dim == 128)
    hipLaunchKernelGGL(k_attn_flash<128>, grid, dim3(WG), 0, st, c->p_qh, c->p_ql, c->p_kc, c->p_vt, c->p_ah, c->p_al, T, c->p_tp,
                       d.n_q_heads, d.n_kv_heads);
  else
    hipLaunchKernelGGL(k_attn_flash<64>, grid, dim3(WG), 0, st, c->p_qh, c->p_ql, c->p_kc, c->p_vt, c->p_ah, c->p_al, T, c->p_tp,
                       d.n_q_heads, d.n_kv_heads);
}

// Prefill of one sequence: T prompt tokens at ids, all layers, routers scored on the way.
template <typename WT>
int prefill_one(first_ctx* c, int b, const int* ids, int T, float* hidden_out, float* logits_out, int* token_out,
                bool soft = false) {
  const first_model_desc& d = c->d;
  hipStream_t st = c->stream;
  const int D = d.d_model, F = d.d_ffn, L = d.n_layers, hd = d.head_dim, P = d.kv_page_tokens;
  const int* pt = c->d_page_table + (size_t)b * c->max_pages;
  const int QB = std::max(1, 64 / c->G);
  const float qscale = 1.0f / std::sqrt((float)hd);
  const size_t kpitch = (size_t)hd * sizeof(WT) + 4;
  const size_t lds_attn = (size_t)64 * hd * sizeof(float) + 64 * kpitch + (size_t)64 * hd * sizeof(WT);
  // activations stay fp32 between the kernels; the bf16 GEMM splits them into two bf16 parts
  float* x = reinterpret_cast<float*>(c->p_x);
  float* a = reinterpret_cast<float*>(c->p_a);
  float* z = reinterpret_cast<float*>(c->p_z);

  hipLaunchKernelGGL(k_embed_rows<WT>, dim3(T), dim3(WG), 0, st, ids, reinterpret_cast<const WT*>(c->embed), c->p_H, D,
                     d.vocab);
  hipLaunchKernelGGL(k_rope_table, dim3((T * c->half + WG - 1) / WG), dim3(WG), 0, st, c->d_theta, c->p_cs, T, c->half);
  for (int i = 0; i < L; ++i) {
    const LayerPtrs& l = c->layers[i];
    // router i reads the stream entering layer i, in the same pass as the attention norm
    const bool hl = d.dtype == FIRST_DTYPE_BF16;   // activations leave their producers split for the matrix cores
    hipLaunchKernelGGL(k_rmsnorm_router<float>, dim3((T + WAVES - 1) / WAVES), dim3(WG), 0, st, c->p_H, l.g_attn,
                       c->router + (size_t)i * D, x, c->p_sig, T, D, d.rms_eps, hl ? c->p_xh : nullptr, hl ? c->p_xl : nullptr);
    hipLaunchKernelGGL(k_router_reduce, dim3(1), dim3(WG), 0, st, c->p_sig, T, c->d_rho + (size_t)b * L + i,
                       c->d_mask + (size_t)b * L + i);
    if (soft)            // the stream entering the layer, for H = Hprev + rho (phi(Hprev))
      HIPCHK(c, hipMemcpyAsync(c->p_Hs, c->p_H, (size_t)T * D * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (c->kv_elide && !soft) {   // the decision is known before the layer stores anything (Section 4.1): fetch it while Q/K/V run
      HIPCHK(c, hipMemcpyAsync(c->h_keep, c->d_mask + (size_t)b * L + i, 1, hipMemcpyDeviceToHost, st));
      HIPCHK(c, hipEventRecord(c->ev_keep, st));
    }
    int rc;
    auto gemm = [&](const float* A32, const bf16* Ah, const bf16* Al, const void* W, float* C, int N, int K, int acc) {
      return hl ? launch_gemm_hl(c, st, Ah, Al, W, C, T, N, K, acc) : launch_gemm(c, st, d.dtype, A32, W, C, T, N, K, acc, true);
    };
    if (hl) {
      if ((rc = launch_gemm_hl_seg(c, st, c->p_xh, c->p_xl, T, D, 0,
                                   {GemmSeg{(const bf16*)l.wq, c->p_q, c->nq, 0}, GemmSeg{(const bf16*)l.wk, c->p_k, c->nkv, 0},
                                    GemmSeg{(const bf16*)l.wv, c->p_v, c->nkv, 0}})))
        return rc;
    } else {
      if ((rc = gemm(x, c->p_xh, c->p_xl, l.wq, c->p_q, c->nq, D, 0))) return rc;
      if ((rc = gemm(x, c->p_xh, c->p_xl, l.wk, c->p_k, c->nkv, D, 0))) return rc;
      if ((rc = gemm(x, c->p_xh, c->p_xl, l.wv, c->p_v, c->nkv, D, 0))) return rc;
    }
    if (c->kv_elide && !soft) {
      HIPCHK(c, hipEventSynchronize(c->ev_keep));
      if (*c->h_keep && c->layer_slice[i] < 0) {
        if (c->slices_used >= c->kv_slots)
          return fail(c, FIRST_ERR_CAPACITY, "first_prefill_route: the routers keep more layers than kv_layer_slots");
        c->layer_slice[i] = c->slices_used++;
      }
    }
    c->has_kv[b][i] = c->layer_slice[i] >= 0;
    WT* pool = reinterpret_cast<WT*>(kv_base(c, i));   // a layer without a slice lends its prompt K/V to the scratch slice
    hipLaunchKernelGGL(k_rope_kvwrite<WT>, dim3(T), dim3(WG), 0, st, c->p_q, c->p_k, c->p_v, c->p_cs, pt, pool,
                       c->page_elems, d.n_q_heads, d.n_kv_heads, hd, P, qscale);
    if (c->p_qh && c->prefill_flash) {
      launch_attn_flash(c, st, reinterpret_cast<const bf16*>(pool), pt, T);
    } else {
      hipLaunchKernelGGL((k_attn_prefill<float, WT>), dim3((T + QB - 1) / QB, d.n_kv_heads), dim3(WG), lds_attn, st, c->p_q, a,
                         pt, pool, c->page_elems, T, d.n_q_heads, d.n_kv_heads, hd, P, QB);
      if (hl) {
        const size_t n = (size_t)T * c->nq;
        hipLaunchKernelGGL(k_split_bf16, dim3((unsigned)std::min<size_t>((n + WG - 1) / WG, 16384)), dim3(WG), 0, st, a, c->p_ah,
                           c->p_al, n);
      }
    }
    if ((rc = gemm(a, c->p_ah, c->p_al, l.wo, c->p_H, D, c->nq, 1))) return rc;
    hipLaunchKernelGGL(k_rmsnorm_router<float>, dim3((T + WAVES - 1) / WAVES), dim3(WG), 0, st, c->p_H, l.g_mlp,
                       (const float*)nullptr, x, (float*)nullptr, T, D, d.rms_eps, hl ? c->p_xh : nullptr, hl ? c->p_xl : nullptr);
    if (hl) {        // SiLU(gate) * up in the GEMM's epilogue, written split for the down projection
      hipLaunchKernelGGL(k_gemm_nt_bf16_hl_gu, dim3((F + GB_N / 2 - 1) / (GB_N / 2), (T + GB_M - 1) / GB_M), dim3(WG), 0, st, c->p_xh,
                         c->p_xl, (const bf16*)l.wg, (const bf16*)l.wu, c->p_zh, c->p_zl, T, F, D);
      HIPCHK(c, hipGetLastError());
    } else {
      if ((rc = gemm(x, c->p_xh, c->p_xl, l.wg, c->p_g, F, D, 0))) return rc;
      if ((rc = gemm(x, c->p_xh, c->p_xl, l.wu, c->p_u, F, D, 0))) return rc;
    }
    const unsigned sm_grid = (unsigned)std::min<size_t>(((size_t)T * F + WG - 1) / WG, 65536);
    if (!hl) hipLaunchKernelGGL(k_silu_mul<float>, dim3(sm_grid), dim3(WG), 0, st, c->p_g, c->p_u, z, (size_t)T * F);
    if ((rc = gemm(z, c->p_zh, c->p_zl, l.wd, c->p_H, D, F, 1))) return rc;
    if (soft)
      hipLaunchKernelGGL(k_soft_blend, dim3((unsigned)std::min<size_t>(((size_t)T * D + WG - 1) / WG, 4096)), dim3(WG), 0, st,
                         c->p_H, c->p_Hs, c->d_rho + (size_t)b * L + i, (size_t)T * D);
  }
  if (soft) {
    HIPCHK(c, hipGetLastError());
    return FIRST_OK;
  }
  // last position -> decode residual slot of this sequence (+ optional copy out), first token
  hipLaunchKernelGGL(k_copy_f32, dim3((D + WG - 1) / WG), dim3(WG), 0, st, c->p_H + (size_t)(T - 1) * D,
                     c->d_h + (size_t)b * D, hidden_out ? hidden_out + (size_t)b * D : nullptr, D);
  hipLaunchKernelGGL(k_set_int, dim3(1), dim3(1), 0, st, c->d_len + b, T);
  DecParams p = base_params(c, b, 1);
  enqueue_head<WT>(c, p, logits_out, token_out, 0);
  HIPCHK(c, hipGetLastError());
  return FIRST_OK;
}

int compact_masks(first_ctx* c) {
  hipLaunchKernelGGL(k_compact, dim3(c->d.max_batch), dim3(64), 0, c->stream, c->d_mask, c->d.n_layers, c->d_kept,
                     c->d_nkept);
  HIPCHK(c, hipGetLastError());
  return FIRST_OK;
}

int alloc_page(first_ctx* c, int b) {
  if (c->free_pages.empty() || c->seq_npages[b] >= c->max_pages) return -1;
  const int pg = c->free_pages.back();
  c->free_pages.pop_back();
  c->h_page_table[(size_t)b * c->max_pages + c->seq_npages[b]] = pg;
  return c->seq_npages[b]++;
}

}  // namespace

extern "C" {

int first_create(const first_model_desc* desc, const first_weights* w, void* hip_stream, first_ctx** out) {
  if (!desc || !w || !out) return fail(nullptr, FIRST_ERR_ARG, "first_create: null argument");
  const first_model_desc& d = *desc;
  if (d.n_layers < 1 || d.d_model < 8 || d.d_model % 8 || d.n_q_heads < 1 || d.n_kv_heads < 1 ||
      d.n_q_heads % d.n_kv_heads || d.n_q_heads / d.n_kv_heads > 8 || (d.head_dim != 64 && d.head_dim != 128) ||
      d.d_ffn < 8 || d.d_ffn % 8 || d.vocab < 1 || (d.dtype != FIRST_DTYPE_FP32 && d.dtype != FIRST_DTYPE_BF16) ||
      d.kv_page_tokens < 1 || d.kv_layer_slots < 0 || d.max_batch < 1 || d.max_seq_len < 2 || !(d.rope_base > 0.f) || !(d.rms_eps >= 0.f))
    return fail(nullptr, FIRST_ERR_ARG, "first_create: unsupported model geometry");
  if (!w->embed || !w->lm_head || !w->final_norm || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo ||
      !w->mlp_norm || !w->w_gate || !w->w_up || !w->w_down || !w->router)
    return fail(nullptr, FIRST_ERR_ARG, "first_create: null weight pointer");
  first_ctx* c = new first_ctx();
  c->d = d;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  if (!c->stream) {
    // graphs cannot be captured on the null stream: use a private stream that keeps the
    // null stream's implicit ordering (created without the non-blocking flag)
    if (hipStreamCreateWithFlags(&c->stream, hipStreamDefault) != hipSuccess) {
      delete c;
      return fail(nullptr, FIRST_ERR_HIP, "first_create: hipStreamCreate failed");
    }
    c->own_stream = true;
  }
  c->num_cu = device_cus();
  c->embed = w->embed; c->lm_head = w->lm_head; c->g_final = w->final_norm; c->router = w->router;
  c->layers.resize(d.n_layers);
  for (int i = 0; i < d.n_layers; ++i) {
    LayerPtrs& l = c->layers[i];
    l.wq = w->wq[i]; l.wk = w->wk[i]; l.wv = w->wv[i]; l.wo = w->wo[i];
    l.wg = w->w_gate[i]; l.wu = w->w_up[i]; l.wd = w->w_down[i];
    l.g_attn = w->attn_norm[i]; l.g_mlp = w->mlp_norm[i];
    if (!l.wq || !l.wk || !l.wv || !l.wo || !l.wg || !l.wu || !l.wd || !l.g_attn || !l.g_mlp) {
      if (c->own_stream) (void)hipStreamDestroy(c->stream);
      delete c;
      return fail(nullptr, FIRST_ERR_ARG, "first_create: null layer weight pointer");
    }
  }
  c->nq = d.n_q_heads * d.head_dim; c->nkv = d.n_kv_heads * d.head_dim; c->half = d.head_dim / 2;
  c->G = d.n_q_heads / d.n_kv_heads;
  c->elem = d.dtype == FIRST_DTYPE_BF16 ? 2 : 4;
  c->max_pages = (d.max_seq_len + d.kv_page_tokens - 1) / d.kv_page_tokens;
  c->n_pages = c->max_pages * d.max_batch;
  c->page_elems = (size_t)2 * d.n_kv_heads * d.kv_page_tokens * d.head_dim;

  const int B = d.max_batch, L = d.n_layers, T = d.max_seq_len;
  int rc = FIRST_OK;
  auto A = [&](int r) { if (rc == FIRST_OK) rc = r; };
  c->kv_elide = d.kv_layer_slots > 0 && d.kv_layer_slots < L;
  c->kv_slots = c->kv_elide ? d.kv_layer_slots : L;
  c->has_kv.assign(B, std::vector<uint8_t>(L, 0));
  reset_layer_slices(c);
  A(dev_alloc(c, &c->kv_pool, (size_t)(c->kv_slots + (c->kv_elide ? 1 : 0)) * kv_slice_bytes(c)));
  if (c->kv_elide && rc == FIRST_OK) {
    if (hipHostMalloc(reinterpret_cast<void**>(&c->h_keep), 64, hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_keep, hipEventDisableTiming) != hipSuccess)
      rc = fail(c, FIRST_ERR_HIP, "first_create: pinned byte / event for the router decisions");
  }
  A(dev_alloc(c, &c->d_page_table, (size_t)B * c->max_pages));
  A(dev_alloc(c, &c->d_len, B)); A(dev_alloc(c, &c->d_kept, (size_t)B * L)); A(dev_alloc(c, &c->d_nkept, B));
  A(dev_alloc(c, &c->d_mask, (size_t)B * L)); A(dev_alloc(c, &c->d_rho, (size_t)B * L));
  A(dev_alloc(c, &c->d_theta, c->half));
  A(dev_alloc(c, &c->d_h, (size_t)B * d.d_model)); A(dev_alloc(c, &c->d_qkv, (size_t)B * (c->nq + 2 * c->nkv)));
  A(dev_alloc(c, &c->d_attn, (size_t)B * c->nq)); A(dev_alloc(c, &c->d_z, (size_t)B * d.d_ffn));
  A(dev_alloc(c, &c->d_part_o, (size_t)B * d.n_q_heads * S_MAX * d.head_dim));
  A(dev_alloc(c, &c->d_part_ml, (size_t)B * d.n_q_heads * S_MAX * 2));
  A(dev_alloc(c, &c->d_attn_cnt, (size_t)B * d.n_kv_heads)); A(dev_alloc(c, &c->d_head_cnt, B));
  A(dev_alloc(c, &c->d_rope_cs, (size_t)B * c->half)); A(dev_alloc(c, &c->d_arg_part, (size_t)B * ARG_MAX_WG));
  A(dev_alloc(c, &c->p_H, (size_t)T * d.d_model)); A(dev_alloc(c, &c->p_q, (size_t)T * c->nq));
  A(dev_alloc(c, &c->p_k, (size_t)T * c->nkv)); A(dev_alloc(c, &c->p_v, (size_t)T * c->nkv));
  if (d.dtype != FIRST_DTYPE_BF16) {   // (bf16 models form SiLU(gate) * up in the GEMM's epilogue: no fp32 gate / up matrices)
    A(dev_alloc(c, &c->p_g, (size_t)T * d.d_ffn)); A(dev_alloc(c, &c->p_u, (size_t)T * d.d_ffn));
  }
  A(dev_alloc(c, &c->p_sig, T)); A(dev_alloc(c, &c->p_cs, (size_t)T * c->half));
  A(dev_alloc(c, reinterpret_cast<char**>(&c->p_x), (size_t)T * d.d_model * 4));
  A(dev_alloc(c, reinterpret_cast<char**>(&c->p_a), (size_t)T * c->nq * 4));
  if (d.dtype == FIRST_DTYPE_BF16) {
    A(dev_alloc(c, &c->p_xh, (size_t)T * d.d_model)); A(dev_alloc(c, &c->p_xl, (size_t)T * d.d_model));
    A(dev_alloc(c, &c->p_ah, (size_t)T * c->nq)); A(dev_alloc(c, &c->p_al, (size_t)T * c->nq));
    A(dev_alloc(c, &c->p_zh, (size_t)T * d.d_ffn)); A(dev_alloc(c, &c->p_zl, (size_t)T * d.d_ffn));
  }
  c->p_tp = (T + FA_KT - 1) / FA_KT * FA_KT;
  if (d.dtype == FIRST_DTYPE_BF16 && (d.head_dim == 64 || d.head_dim == 128)) {
    A(dev_alloc(c, &c->p_qh, (size_t)T * c->nq)); A(dev_alloc(c, &c->p_ql, (size_t)T * c->nq));
    A(dev_alloc(c, &c->p_kc, (size_t)c->p_tp * c->nkv)); A(dev_alloc(c, &c->p_vt, (size_t)c->p_tp * c->nkv));
  }
  A(dev_alloc(c, reinterpret_cast<char**>(&c->p_z), (size_t)T * d.d_ffn * 4));
  c->xpitch = (std::max(std::max(d.d_model, c->nq), d.d_ffn) + 31) / 32 * 32;
  if (B > 1) {
    A(dev_alloc(c, &c->d_xh, (size_t)BATCH_SLOTS * c->xpitch)); A(dev_alloc(c, &c->d_xl, (size_t)BATCH_SLOTS * c->xpitch));
    A(dev_alloc(c, &c->d_zh, (size_t)BATCH_SLOTS * c->xpitch)); A(dev_alloc(c, &c->d_zl, (size_t)BATCH_SLOTS * c->xpitch));
    A(dev_alloc(c, &c->d_rinv, BATCH_SLOTS)); A(dev_alloc(c, &c->d_logits_all, (size_t)B * d.vocab));
    {                                                   // partial sums: up to 8 slices x 16 slots x (rows padded to a tile group), gate + up
      const size_t nmax = (size_t)std::max(std::max(c->nq + 2 * c->nkv, d.d_model), 2 * d.d_ffn);
      c->bg_cnt_n = nmax / (5 * 16) + 2;
      c->bg_part_floats = (size_t)8 * 16 * (nmax + 8 * 16 * 2);
    }
    A(dev_alloc(c, &c->d_bg_part, c->bg_part_floats)); A(dev_alloc(c, &c->d_bg_cnt, c->bg_cnt_n));
    A(dev_alloc(c, &c->d_x2h, (size_t)BATCH_SLOTS * c->xpitch)); A(dev_alloc(c, &c->d_x2l, (size_t)BATCH_SLOTS * c->xpitch));
    A(dev_alloc(c, &c->d_ssq, c->bg_cnt_n * BATCH_SLOTS));
  }
  if (B > 1 && rc == FIRST_OK) {
    (void)hipMemset(c->d_xh, 0, (size_t)BATCH_SLOTS * c->xpitch * 2); (void)hipMemset(c->d_xl, 0, (size_t)BATCH_SLOTS * c->xpitch * 2);
    (void)hipMemset(c->d_zh, 0, (size_t)BATCH_SLOTS * c->xpitch * 2); (void)hipMemset(c->d_zl, 0, (size_t)BATCH_SLOTS * c->xpitch * 2);
    (void)hipMemset(c->d_bg_cnt, 0, c->bg_cnt_n * sizeof(unsigned));
    (void)hipMemset(c->d_x2h, 0, (size_t)BATCH_SLOTS * c->xpitch * 2); (void)hipMemset(c->d_x2l, 0, (size_t)BATCH_SLOTS * c->xpitch * 2);
#define FIRST_BGG_ATTR(MODE)                                                                                          \
  for (const void* fn : {reinterpret_cast<const void*>(&k_bgemv_g<MODE, 8>), reinterpret_cast<const void*>(&k_bgemv_g<MODE, 7>),      \
                         reinterpret_cast<const void*>(&k_bgemv_g<MODE, 6>), reinterpret_cast<const void*>(&k_bgemv_g<MODE, 5>)})      \
    (void)hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    FIRST_BGG_ATTR(BG_QKV) FIRST_BGG_ATTR(BG_O) FIRST_BGG_ATTR(BG_DN) FIRST_BGG_ATTR(BG_GU)
#undef FIRST_BGG_ATTR
  }
  A(dev_alloc(c, &c->d_topk_part, (size_t)B * ((d.vocab + SMP_CHUNK - 1) / SMP_CHUNK) * SMP_KMAX));
  A(dev_alloc(c, &c->d_step_cands, (size_t)c->num_cu * SMP_KMAX));
  A(dev_alloc(c, &c->d_logits_own, (size_t)B * d.vocab));
  A(dev_alloc(c, &c->x_h, (size_t)B * d.d_model)); A(dev_alloc(c, &c->x_qkv, (size_t)B * (c->nq + 2 * c->nkv)));
  A(dev_alloc(c, &c->x_attn, (size_t)B * c->nq)); A(dev_alloc(c, &c->x_z, (size_t)B * d.d_ffn));
  A(dev_alloc(c, &c->x_part, sk_part_index(d.n_q_heads, d.head_dim, B, 0, 0)));
  A(dev_alloc(c, &c->d_tagstate, (size_t)B * 8));
  A(dev_alloc(c, &c->d_layers, L)); A(dev_alloc(c, &c->d_done, (size_t)c->num_cu)); A(dev_alloc(c, &c->d_err, 4));
  A(dev_alloc(c, &c->d_tdbg, (size_t)(4 * L + 1) * SK_TSLOTS));
  if (rc == FIRST_OK) {
    std::vector<double> theta(c->half);
    for (int i = 0; i < c->half; ++i) theta[i] = std::pow((double)d.rope_base, -2.0 * i / d.head_dim);
    hipError_t e = hipMemcpy(c->d_theta, theta.data(), c->half * sizeof(double), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(c->d_attn_cnt, 0, (size_t)B * d.n_kv_heads * sizeof(unsigned));
    if (e == hipSuccess) e = hipMemset(c->d_head_cnt, 0, B * sizeof(unsigned));
    if (e == hipSuccess) e = hipMemset(c->d_len, 0, B * sizeof(int));
    if (e == hipSuccess) e = hipMemset(c->d_err, 0, 4 * sizeof(int));
    if (e == hipSuccess) e = reset_tagged_exchange(c);
    c->step_ok = step_kernel_fits(c);
    if (e == hipSuccess && c->step_ok) {
      e = make_permuted_down_copies(c);
      if (e == hipSuccess) e = upload_layer_table(c);
      c->step_lds = sk_lds_floats(d.d_model, c->nq, d.d_ffn, c->G, d.head_dim) * sizeof(float);
      const void* fn = step_kernel_fn(c);
      if (e == hipSuccess) e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->step_lds);
      int per_cu = 0;
      if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, SK_THREADS, c->step_lds);
      if (e == hipSuccess && per_cu < 1) c->step_ok = false;   // grid would not be co-resident
    }
    if (e == hipSuccess && B > 1 && d.dtype == FIRST_DTYPE_BF16 && d_batch_fits(c)) e = make_tiled_copies(c);
    if (e == hipSuccess) e = hipMemset(c->d_mask, 0, (size_t)B * L);
    if (e == hipSuccess) e = hipMemset(c->d_page_table, 0, (size_t)B * c->max_pages * sizeof(int));
    // the prefill attention kernels stage more than 64 KB of LDS for head_dim 128
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_prefill<float, bf16>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_prefill<float, float>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    if (e != hipSuccess) rc = fail(nullptr, FIRST_ERR_HIP, std::string("first_create: ") + hipGetErrorString(e));
  } else {
    g_create_error = c->err;
  }
  if (rc != FIRST_OK) {
    for (void* p : c->allocs) (void)hipFree(p);
    if (c->h_keep) (void)hipHostFree(c->h_keep);
    if (c->ev_keep) (void)hipEventDestroy(c->ev_keep);
    if (c->own_stream) (void)hipStreamDestroy(c->stream);
    delete c;
    return rc;
  }
  c->hlen.assign(B, 0); c->decoded.assign(B, 0); c->seq_npages.assign(B, 0);
  c->hmask.assign(B, std::vector<uint8_t>(L, 0));
  c->h_page_table.assign((size_t)B * c->max_pages, 0);
  c->page_order.resize(c->n_pages);
  for (int i = 0; i < c->n_pages; ++i) c->page_order[i] = i;
  release_sequences(c);
  *out = c;
  return FIRST_OK;
}

int first_destroy(first_ctx* c) {
  if (!c) return FIRST_ERR_ARG;
  (void)hipStreamSynchronize(c->stream);
  drop_graphs(c);
  for (void* p : c->allocs) (void)hipFree(p);
  if (c->h_keep) (void)hipHostFree(c->h_keep);
  if (c->ev_keep) (void)hipEventDestroy(c->ev_keep);
  if (c->own_stream) (void)hipStreamDestroy(c->stream);
  delete c;
  return FIRST_OK;
}

int first_prefill_route(first_ctx* c, int32_t B, const int32_t* ids, const int32_t* lens, float* rho_out,
                        uint8_t* mask_out, float* hidden_out, float* logits_out, int32_t* token_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!ids || !lens) return fail(c, FIRST_ERR_ARG, "first_prefill_route: null ids/lens");
  if (B < 1 || B > c->d.max_batch) return fail(c, FIRST_ERR_CAPACITY, "first_prefill_route: batch exceeds max_batch");
  for (int b = 0; b < B; ++b) {
    if (lens[b] < 1) return fail(c, FIRST_ERR_ARG, "first_prefill_route: empty prompt");
    if (lens[b] >= c->d.max_seq_len)
      return fail(c, FIRST_ERR_CAPACITY, "first_prefill_route: prompt does not leave room for a generated token");
  }
  const int L = c->d.n_layers, P = c->d.kv_page_tokens;
  release_sequences(c);
  drop_graphs(c);
  // pages for every prompt, then one upload of the page tables
  for (int b = 0; b < B; ++b)
    for (int need = (lens[b] + P - 1) / P; c->seq_npages[b] < need;)
      if (alloc_page(c, b) < 0) return fail(c, FIRST_ERR_CAPACITY, "first_prefill_route: out of KV pages");
  HIPCHK(c, hipMemcpyAsync(c->d_page_table, c->h_page_table.data(), c->h_page_table.size() * sizeof(int),
                           hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));     // the host table may now be edited again
  size_t off = 0;
  for (int b = 0; b < B; ++b) {
    const int rc = c->d.dtype == FIRST_DTYPE_BF16
                       ? prefill_one<bf16>(c, b, ids + off, lens[b], hidden_out, logits_out, token_out)
                       : prefill_one<float>(c, b, ids + off, lens[b], hidden_out, logits_out, token_out);
    if (rc) return rc;
    off += lens[b];
    c->hlen[b] = lens[b];
  }
  c->B = B;
  int rc = compact_masks(c);
  if (rc) return rc;
  std::vector<uint8_t> hm((size_t)B * L);
  HIPCHK(c, hipMemcpyAsync(hm.data(), c->d_mask, hm.size(), hipMemcpyDeviceToHost, c->stream));
  if (rho_out) HIPCHK(c, hipMemcpyAsync(rho_out, c->d_rho, (size_t)B * L * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
  if (mask_out) HIPCHK(c, hipMemcpyAsync(mask_out, c->d_mask, (size_t)B * L, hipMemcpyDeviceToDevice, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  for (int b = 0; b < B; ++b) c->hmask[b].assign(hm.begin() + (size_t)b * L, hm.begin() + (size_t)(b + 1) * L);
  if (c->kv_elide && c->step_ok) HIPCHK(c, upload_layer_table(c));   // the layers' slices are new
  return FIRST_OK;
}

int first_set_mask(first_ctx* c, int32_t seq, const uint8_t* mask) {
  if (!c) return FIRST_ERR_ARG;
  if (!mask) return fail(c, FIRST_ERR_ARG, "first_set_mask: null mask");
  if (seq < 0 || seq >= c->B) return fail(c, FIRST_ERR_STATE, "first_set_mask: no such live sequence");
  const int L = c->d.n_layers;
  std::vector<uint8_t> m(L);
  for (int i = 0; i < L; ++i) {
    m[i] = mask[i] ? 1 : 0;
    if (c->decoded[seq] && m[i] && !c->hmask[seq][i])
      return fail(c, FIRST_ERR_STATE, "first_set_mask: layer was skipped by earlier decode tokens; its KV has holes");
    if (m[i] && !c->has_kv[seq][i])
      return fail(c, FIRST_ERR_STATE, "first_set_mask: the prompt KV of this layer was not stored (kv_layer_slots)");
  }
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(c->d_mask + (size_t)seq * L, m.data(), L, hipMemcpyHostToDevice));
  c->hmask[seq] = m;
  return compact_masks(c);
}

int first_get_kept(first_ctx* c, int32_t seq, int32_t* kept_idx, int32_t* n_kept) {
  if (!c) return FIRST_ERR_ARG;
  if (!kept_idx || !n_kept) return fail(c, FIRST_ERR_ARG, "first_get_kept: null output");
  if (seq < 0 || seq >= c->B) return fail(c, FIRST_ERR_STATE, "first_get_kept: no such live sequence");
  const int L = c->d.n_layers;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(kept_idx, c->d_kept + (size_t)seq * L, L * sizeof(int), hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(n_kept, c->d_nkept + seq, sizeof(int), hipMemcpyDeviceToHost));
  return check_step_error(c, "first_get_kept");
}

namespace {
// One decode step, greedy (smp null) or with the paper's decoding rule.  On the persistent kernel the rule is part of the
// kernel's LM-head epilogue; elsewhere the step's logits go through the two sampling kernels.
int decode_step_impl(first_ctx* c, const int32_t* last_tokens, float* logits_out, int32_t* token_out, const SampleArgs* smp) {
  if (c->B < 1) return fail(c, FIRST_ERR_STATE, "first_decode_step: no prefilled sequence");
  const int P = c->d.kv_page_tokens;
  int max_len = 0;
  for (int b = 0; b < c->B; ++b) {
    if (c->hlen[b] + 1 > c->d.max_seq_len) return fail(c, FIRST_ERR_CAPACITY, "first_decode_step: sequence is full");
    max_len = std::max(max_len, c->hlen[b]);
  }
  int S = c->attn_splits;
  if (S <= 0) S = (max_len + 128 + 127) / 128;
  S = std::max(1, std::min(S, 32));
  const bool bf = c->d.dtype == FIRST_DTYPE_BF16;
  const bool persistent = c->step_ok && c->B == 1 && c->decode_path != 0;
  if (c->decode_path == 1 && !persistent)
    return fail(c, FIRST_ERR_STATE, "first_decode_step: the persistent kernel needs a bf16 model whose widths are "
                                    "multiples of 256, 16-token pages and exactly one live sequence");
  const bool batch_ok = bf && c->B > 1 && c->d_xh && d_batch_fits(c);
  const bool batched = !persistent && batch_ok && c->batch_path != 0;
  // (the persistent kernel merges the workgroups' candidate lists in LDS: a large top_k may not fit there)
  const bool fused = smp && persistent && smp->top_k <= sk_sample_kmax(c->d.d_model, c->nq, c->d.d_ffn, c->num_cu);
  if (smp && !fused && !logits_out) logits_out = c->d_logits_own;
  if (c->batch_path == 1 && !persistent && !batched)
    return fail(c, FIRST_ERR_STATE, "first_decode_step: the batched path needs a bf16 model whose widths are multiples of 8 "
                                    "and more than one live sequence");
  // the page that will receive position len[b] must exist: count what is missing before handing anything out, so
  // that a refusal leaves every sequence as it was
  {
    int need = 0;
    for (int b = 0; b < c->B; ++b)
      if (c->hlen[b] / P >= c->seq_npages[b]) {
        if (c->seq_npages[b] >= c->max_pages) return fail(c, FIRST_ERR_CAPACITY, "first_decode_step: out of KV pages");
        ++need;
      }
    if (need > (int)c->free_pages.size()) return fail(c, FIRST_ERR_CAPACITY, "first_decode_step: out of KV pages");
  }
  for (int b = 0; b < c->B; ++b) {
    if (c->hlen[b] / P >= c->seq_npages[b]) {
      const int slot = alloc_page(c, b);
      hipLaunchKernelGGL(k_set_int, dim3(1), dim3(1), 0, c->stream, c->d_page_table + (size_t)b * c->max_pages + slot,
                         c->h_page_table[(size_t)b * c->max_pages + slot]);
    }
  }
  auto enqueue = [&]() {
    if (persistent) enqueue_decode_step_kernel(c, last_tokens, logits_out, token_out, fused ? smp : nullptr);
    else if (batched) enqueue_decode_batched(c, last_tokens, logits_out, token_out, S);
    else if (bf) enqueue_decode_ops<bf16>(c, last_tokens, logits_out, token_out, S);
    else enqueue_decode_ops<float>(c, last_tokens, logits_out, token_out, S);
    if (smp && !fused) {
      const int chunks = (c->d.vocab + SMP_CHUNK - 1) / SMP_CHUNK;
      hipLaunchKernelGGL(k_topk_part, dim3(chunks, c->B), dim3(SMP_THREADS), 0, c->stream, logits_out, c->d.vocab, smp->top_k, c->d_topk_part);
      hipLaunchKernelGGL(k_topk_sample, dim3(c->B), dim3(SMP_THREADS), 0, c->stream, c->d_topk_part, chunks * smp->top_k, smp->top_k,
                         smp->temperature, smp->uniforms, token_out, smp->candidates_out);
    }
  };
  if (!c->use_graph) {
    enqueue();
    HIPCHK(c, hipGetLastError());
  } else {
    // the persistent kernel reads the kept list from the device: one graph whatever the mask
    const int kind = persistent ? -1 : batched ? S + 1000 : S;
    std::string key(reinterpret_cast<const char*>(&kind), sizeof(kind));
    key.append(reinterpret_cast<const char*>(&last_tokens), sizeof(void*));
    key.append(reinterpret_cast<const char*>(&logits_out), sizeof(void*));
    key.append(reinterpret_cast<const char*>(&token_out), sizeof(void*));
    if (smp) key.append(reinterpret_cast<const char*>(smp), sizeof(*smp));      // (pointers and values are part of the captured arguments)
    if (!persistent)
      for (int b = 0; b < c->B; ++b) key.append(reinterpret_cast<const char*>(c->hmask[b].data()), c->hmask[b].size());
    auto it = c->graphs.find(key);
    if (it == c->graphs.end()) {
      if (c->graphs.size() >= 32) {
        // make room for one: the least recently used entry goes (it may still be running: wait first)
        auto old = c->graphs.begin();
        for (auto g = c->graphs.begin(); g != c->graphs.end(); ++g)
          if (g->second.used < old->second.used) old = g;
        HIPCHK(c, hipStreamSynchronize(c->stream));
        (void)hipGraphExecDestroy(old->second.exec);
        c->graphs.erase(old);
      }
      hipGraph_t graph = nullptr;
      hipGraphExec_t exec = nullptr;
      HIPCHK(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
      enqueue();
      const hipError_t e_launch = hipGetLastError();
      const hipError_t e_end = hipStreamEndCapture(c->stream, &graph);      // (also what abandons a capture that went wrong)
      if (e_launch != hipSuccess || e_end != hipSuccess) {
        if (graph) (void)hipGraphDestroy(graph);
        return fail(c, FIRST_ERR_HIP, std::string("first_decode_step: graph capture: ") +
                                          hipGetErrorString(e_launch != hipSuccess ? e_launch : e_end));
      }
      const hipError_t e_inst = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
      (void)hipGraphDestroy(graph);
      if (e_inst != hipSuccess)
        return fail(c, FIRST_ERR_HIP, std::string("first_decode_step: hipGraphInstantiate: ") + hipGetErrorString(e_inst));
      it = c->graphs.emplace(key, first_ctx::CachedGraph{exec, 0}).first;
    }
    it->second.used = ++c->graph_clock;
    HIPCHK(c, hipGraphLaunch(it->second.exec, c->stream));
  }
  for (int b = 0; b < c->B; ++b) { c->hlen[b] += 1; c->decoded[b] = 1; }
  return FIRST_OK;
}
}  // namespace

int first_decode_step(first_ctx* c, const int32_t* last_tokens, float* logits_out, int32_t* token_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!last_tokens) return fail(c, FIRST_ERR_ARG, "first_decode_step: null tokens");
  return decode_step_impl(c, last_tokens, logits_out, token_out, nullptr);
}

int first_decode_step_sampled(first_ctx* c, const int32_t* last_tokens, const float* uniforms, float temperature, int32_t top_k,
                              float* logits_out, int32_t* token_out, int32_t* candidates_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!last_tokens || !uniforms || !token_out) return fail(c, FIRST_ERR_ARG, "first_decode_step_sampled: null pointer");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return fail(c, FIRST_ERR_ARG, "first_decode_step_sampled: temperature must be positive");
  if (top_k < 1 || top_k > SMP_KMAX) return fail(c, FIRST_ERR_ARG, "first_decode_step_sampled: top_k must be in 1..64");
  SampleArgs smp{};                                  // (zeroed: the struct's bytes are part of the graph key)
  smp.uniforms = uniforms; smp.temperature = temperature; smp.top_k = top_k; smp.candidates_out = candidates_out;
  return decode_step_impl(c, last_tokens, logits_out, token_out, &smp);
}

int first_sample_top_k(first_ctx* c, const float* logits, const float* uniforms, float temperature, int32_t top_k,
                       int32_t* token_out, int32_t* candidates_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!logits || !uniforms || !token_out) return fail(c, FIRST_ERR_ARG, "first_sample_top_k: null pointer");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return fail(c, FIRST_ERR_ARG, "first_sample_top_k: temperature must be positive");
  if (top_k < 1 || top_k > SMP_KMAX) return fail(c, FIRST_ERR_ARG, "first_sample_top_k: top_k must be in 1..64");
  if (c->B < 1) return fail(c, FIRST_ERR_STATE, "first_sample_top_k: no live sequence");
  const int chunks = (c->d.vocab + SMP_CHUNK - 1) / SMP_CHUNK;
  hipLaunchKernelGGL(k_topk_part, dim3(chunks, c->B), dim3(SMP_THREADS), 0, c->stream, logits, c->d.vocab, top_k, c->d_topk_part);
  hipLaunchKernelGGL(k_topk_sample, dim3(c->B), dim3(SMP_THREADS), 0, c->stream, c->d_topk_part, chunks * top_k, top_k,
                     temperature, uniforms, token_out, candidates_out);
  HIPCHK(c, hipGetLastError());
  return FIRST_OK;
}

int first_sample_top_k_static(void* hip_stream, const float* logits, int32_t n_seq, int32_t vocab, const float* uniforms,
                              float temperature, int32_t top_k, int32_t* token_out, int32_t* candidates_out) {
  auto bad = [](int code, const char* msg) { g_create_error = msg; return code; };
  if (!logits || !uniforms || !token_out) return bad(FIRST_ERR_ARG, "first_sample_top_k_static: null pointer");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return bad(FIRST_ERR_ARG, "first_sample_top_k_static: temperature must be positive");
  if (top_k < 1 || top_k > SMP_KMAX) return bad(FIRST_ERR_ARG, "first_sample_top_k_static: top_k must be in 1..64");
  if (n_seq < 1 || vocab < 1) return bad(FIRST_ERR_ARG, "first_sample_top_k_static: n_seq and vocab must be positive");
  const long long chunks = ((long long)vocab + SMP_CHUNK - 1) / SMP_CHUNK;
  if ((long long)n_seq * chunks * top_k > STATIC_SCRATCH_CANDS || chunks > 65535 || n_seq > 65535)
    return bad(FIRST_ERR_CAPACITY, "first_sample_top_k_static: n_seq * ceil(vocab / 2048) * top_k exceeds the 131072 candidates "
                                   "of the static scratch array");
  Cand* part = nullptr;
  {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_SCRATCH_MAX_DEV)
      return bad(FIRST_ERR_HIP, "first_sample_top_k_static: no current device (or device ordinal >= 64)");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {                       // once per device: the address of THIS device's copy of the array
      void* p = nullptr;
      const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p) {
        g_create_error = std::string("first_sample_top_k_static: hipGetSymbolAddress: ") + hipGetErrorString(e);
        return FIRST_ERR_HIP;
      }
      g_scratch_ptr[dev] = p;
    }
    part = reinterpret_cast<Cand*>(g_scratch_ptr[dev]);
  }
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  // every candidate slot stage 2 reads is written by stage 1 of the same call: nothing to clear
  hipLaunchKernelGGL(k_topk_part, dim3((unsigned)chunks, n_seq), dim3(SMP_THREADS), 0, st, logits, vocab, top_k, part);
  hipLaunchKernelGGL(k_topk_sample, dim3(n_seq), dim3(SMP_THREADS), 0, st, part, (int)chunks * top_k, top_k, temperature, uniforms,
                     token_out, candidates_out);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    g_create_error = std::string("first_sample_top_k_static: ") + hipGetErrorString(e);
    return FIRST_ERR_HIP;
  }
  return FIRST_OK;
}

int first_set_option(first_ctx* c, int32_t option, int32_t value) {
  if (!c) return FIRST_ERR_ARG;
  switch (option) {
    case FIRST_OPT_USE_GRAPH: c->use_graph = value ? 1 : 0; return FIRST_OK;
    case FIRST_OPT_ATTN_SPLITS:
      if (value < 0 || value > S_MAX) return fail(c, FIRST_ERR_ARG, "first_set_option: splits out of range");
      c->attn_splits = value; return FIRST_OK;
    case FIRST_OPT_DECODE_PATH:
      if (value < -1 || value > 1) return fail(c, FIRST_ERR_ARG, "first_set_option: unknown decode path");
      c->decode_path = value; return FIRST_OK;
    case FIRST_OPT_STEP_TIMING:
      c->step_timing = value ? 1 : 0;
      drop_graphs(c);
      return FIRST_OK;
    case FIRST_OPT_BATCH_TILED:
      c->tiled = value != 0 && c->t_head != nullptr;
      drop_graphs(c);
      return FIRST_OK;
    case FIRST_OPT_PREFILL_ATTN:
      c->prefill_flash = value ? 1 : 0; return FIRST_OK;
    case FIRST_OPT_BATCH_PATH:
      if (value < -1 || value > 1) return fail(c, FIRST_ERR_ARG, "first_set_option: unknown batch path");
      c->batch_path = value; return FIRST_OK;
    case FIRST_OPT_STEP_POLL_LIMIT: {
      if (value < -1 || value > (1 << 29)) return fail(c, FIRST_ERR_ARG, "first_set_option: poll limit out of range");
      HIPCHK(c, hipStreamSynchronize(c->stream));
      const int word = value < 0 ? 0 : (value + 1) << 1;
      HIPCHK(c, hipMemcpy(c->d_err, &word, sizeof(int), hipMemcpyHostToDevice));
      return FIRST_OK;
    }
    default: return fail(c, FIRST_ERR_ARG, "first_set_option: unknown option");
  }
}

int first_sync(first_ctx* c) {
  if (!c) return FIRST_ERR_ARG;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return check_step_error(c, "first_sync");
}

const char* first_last_error(const first_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

int first_seq_len(first_ctx* c, int32_t seq, int32_t* len_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!len_out) return fail(c, FIRST_ERR_ARG, "first_seq_len: null output");
  if (seq < 0 || seq >= c->B) return fail(c, FIRST_ERR_STATE, "first_seq_len: no such live sequence");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(len_out, c->d_len + seq, sizeof(int), hipMemcpyDeviceToHost));
  return check_step_error(c, "first_seq_len");
}

int first_batch(first_ctx* c, int32_t* batch_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!batch_out) return fail(c, FIRST_ERR_ARG, "first_batch: null output");
  *batch_out = c->B;
  return FIRST_OK;
}

static int kv_tap(first_ctx* c, int seq, int layer, int pos0, int n, float* k, float* v, bool write) {
  if (!c) return FIRST_ERR_ARG;
  if (!k || !v) return fail(c, FIRST_ERR_ARG, "first_kv: null buffer");
  if (seq < 0 || seq >= c->B) return fail(c, FIRST_ERR_STATE, "first_kv: no such live sequence");
  if (layer < 0 || layer >= c->d.n_layers || pos0 < 0 || n < 0 || pos0 + n > c->seq_npages[seq] * c->d.kv_page_tokens)
    return fail(c, FIRST_ERR_ARG, "first_kv: range outside the sequence's pages");
  if (!c->has_kv[seq][layer]) return fail(c, FIRST_ERR_STATE, "first_kv: the KV of this layer was not stored (kv_layer_slots)");
  if (n == 0) return FIRST_OK;
  char* pool = kv_base(c, layer);
  const int* pt = c->d_page_table + (size_t)seq * c->max_pages;
  const first_model_desc& d = c->d;
  if (d.dtype == FIRST_DTYPE_BF16) {
    if (write) hipLaunchKernelGGL((k_kv_tap<bf16, true>), dim3(n), dim3(WG), 0, c->stream, (bf16*)pool, c->page_elems, pt, pos0, d.n_kv_heads, d.head_dim, d.kv_page_tokens, k, v);
    else hipLaunchKernelGGL((k_kv_tap<bf16, false>), dim3(n), dim3(WG), 0, c->stream, (bf16*)pool, c->page_elems, pt, pos0, d.n_kv_heads, d.head_dim, d.kv_page_tokens, k, v);
  } else {
    if (write) hipLaunchKernelGGL((k_kv_tap<float, true>), dim3(n), dim3(WG), 0, c->stream, (float*)pool, c->page_elems, pt, pos0, d.n_kv_heads, d.head_dim, d.kv_page_tokens, k, v);
    else hipLaunchKernelGGL((k_kv_tap<float, false>), dim3(n), dim3(WG), 0, c->stream, (float*)pool, c->page_elems, pt, pos0, d.n_kv_heads, d.head_dim, d.kv_page_tokens, k, v);
  }
  HIPCHK(c, hipGetLastError());
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return check_step_error(c, "first_kv");
}

int first_kv_read(first_ctx* c, int32_t seq, int32_t layer, int32_t pos0, int32_t n, float* k_out, float* v_out) {
  return kv_tap(c, seq, layer, pos0, n, k_out, v_out, false);
}
int first_kv_write(first_ctx* c, int32_t seq, int32_t layer, int32_t pos0, int32_t n, const float* k_in,
                   const float* v_in) {
  return kv_tap(c, seq, layer, pos0, n, const_cast<float*>(k_in), const_cast<float*>(v_in), true);
}

int first_set_seq_len(first_ctx* c, int32_t seq, int32_t len) {
  if (!c) return FIRST_ERR_ARG;
  if (seq < 0 || seq >= c->B) return fail(c, FIRST_ERR_STATE, "first_set_seq_len: no such live sequence");
  if (len < 1 || len + 1 > c->d.max_seq_len) return fail(c, FIRST_ERR_CAPACITY, "first_set_seq_len: length out of range");
  const int P = c->d.kv_page_tokens;
  while (c->seq_npages[seq] * P < len) {
    const int slot = alloc_page(c, seq);
    if (slot < 0) return fail(c, FIRST_ERR_CAPACITY, "first_set_seq_len: out of KV pages");
    hipLaunchKernelGGL(k_set_int, dim3(1), dim3(1), 0, c->stream, c->d_page_table + (size_t)seq * c->max_pages + slot,
                       c->h_page_table[(size_t)seq * c->max_pages + slot]);
  }
  hipLaunchKernelGGL(k_set_int, dim3(1), dim3(1), 0, c->stream, c->d_len + seq, len);
  HIPCHK(c, hipGetLastError());
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->hlen[seq] = len;
  return FIRST_OK;
}

int first_get_hidden(first_ctx* c, float* hidden_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!hidden_out) return fail(c, FIRST_ERR_ARG, "first_get_hidden: null output");
  if (c->B < 1) return fail(c, FIRST_ERR_STATE, "first_get_hidden: no live sequence");
  HIPCHK(c, hipMemcpyAsync(hidden_out, c->d_h, (size_t)c->B * c->d.d_model * sizeof(float), hipMemcpyDeviceToDevice,
                           c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return check_step_error(c, "first_get_hidden");
}

int first_set_page_order(first_ctx* c, const int32_t* perm) {
  if (!c) return FIRST_ERR_ARG;
  if (!perm) return fail(c, FIRST_ERR_ARG, "first_set_page_order: null permutation");
  if (c->B != 0) return fail(c, FIRST_ERR_STATE, "first_set_page_order: sequences are live");
  std::vector<char> seen(c->n_pages, 0);
  for (int i = 0; i < c->n_pages; ++i) {
    if (perm[i] < 0 || perm[i] >= c->n_pages || seen[perm[i]])
      return fail(c, FIRST_ERR_ARG, "first_set_page_order: not a permutation");
    seen[perm[i]] = 1;
  }
  c->page_order.assign(perm, perm + c->n_pages);
  release_sequences(c);
  return FIRST_OK;
}

int first_num_pages(first_ctx* c, int32_t* n_pages_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!n_pages_out) return fail(c, FIRST_ERR_ARG, "first_num_pages: null output");
  *n_pages_out = c->n_pages;
  return FIRST_OK;
}

int first_kv_usage(first_ctx* c, int64_t* pool_bytes, int32_t* layer_slots, int32_t* slots_in_use) {
  if (!c) return FIRST_ERR_ARG;
  if (pool_bytes) *pool_bytes = (int64_t)((size_t)(c->kv_slots + (c->kv_elide ? 1 : 0)) * kv_slice_bytes(c));
  if (layer_slots) *layer_slots = c->kv_slots;
  if (slots_in_use) *slots_in_use = c->slices_used;
  return FIRST_OK;
}

constexpr int SOFT_ROWS = 128;   // positions whose logits are formed at a time in first_soft_forward

int first_soft_forward(first_ctx* c, int32_t B, const int32_t* ids, const int32_t* lens, const int32_t* targets, float lambda,
                       float alpha, float* rho_out, float* terms_out, float* hidden_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!ids || !lens || !targets || !terms_out) return fail(c, FIRST_ERR_ARG, "first_soft_forward: null ids/lens/targets/terms");
  if (B < 1 || B > c->d.max_batch) return fail(c, FIRST_ERR_CAPACITY, "first_soft_forward: batch exceeds max_batch");
  for (int b = 0; b < B; ++b) {
    if (lens[b] < 1) return fail(c, FIRST_ERR_ARG, "first_soft_forward: empty sequence");
    if (lens[b] > c->d.max_seq_len) return fail(c, FIRST_ERR_CAPACITY, "first_soft_forward: sequence longer than max_seq_len");
  }
  const first_model_desc& d = c->d;
  const int L = d.n_layers, P = d.kv_page_tokens, D = d.d_model, V = d.vocab;
  hipStream_t st = c->stream;
  if (!c->p_Hs) {
    int rc = dev_alloc(c, &c->p_Hs, (size_t)d.max_seq_len * D);
    if (rc == FIRST_OK) rc = dev_alloc(c, &c->p_lg, (size_t)SOFT_ROWS * V);
    if (rc == FIRST_OK) rc = dev_alloc(c, &c->p_ce, (size_t)d.max_seq_len);
    if (rc != FIRST_OK) { c->p_Hs = nullptr; return rc; }
  }
  release_sequences(c);
  drop_graphs(c);
  // the layers' own attention reads K/V through the page tables: pages for every sequence, as a prefill would take them
  for (int b = 0; b < B; ++b)
    for (int need = (lens[b] + P - 1) / P; c->seq_npages[b] < need;)
      if (alloc_page(c, b) < 0) return fail(c, FIRST_ERR_CAPACITY, "first_soft_forward: out of KV pages");
  HIPCHK(c, hipMemcpyAsync(c->d_page_table, c->h_page_table.data(), c->h_page_table.size() * sizeof(int),
                           hipMemcpyHostToDevice, st));
  HIPCHK(c, hipStreamSynchronize(st));
  const bool hl = d.dtype == FIRST_DTYPE_BF16;
  size_t off = 0;
  for (int b = 0; b < B; ++b) {
    const int T = lens[b];
    int rc = hl ? prefill_one<bf16>(c, b, ids + off, T, nullptr, nullptr, nullptr, true)
                : prefill_one<float>(c, b, ids + off, T, nullptr, nullptr, nullptr, true);
    if (rc) return rc;
    if (hidden_out)
      HIPCHK(c, hipMemcpyAsync(hidden_out + off * D, c->p_H, (size_t)T * D * sizeof(float), hipMemcpyDeviceToDevice, st));
    // logits of every position = W_lm . RMSNorm(H_L; g_final), SOFT_ROWS positions at a time, then their cross entropy
    float* x = reinterpret_cast<float*>(c->p_x);
    hipLaunchKernelGGL(k_rmsnorm_router<float>, dim3((T + WAVES - 1) / WAVES), dim3(WG), 0, st, c->p_H, c->g_final,
                       (const float*)nullptr, x, (float*)nullptr, T, D, d.rms_eps, hl ? c->p_xh : nullptr, hl ? c->p_xl : nullptr);
    for (int r0 = 0; r0 < T; r0 += SOFT_ROWS) {
      const int rows = std::min(SOFT_ROWS, T - r0);
      rc = hl ? launch_gemm_hl(c, st, c->p_xh + (size_t)r0 * D, c->p_xl + (size_t)r0 * D, c->lm_head, c->p_lg, rows, V, D, 0)
              : launch_gemm(c, st, d.dtype, x + (size_t)r0 * D, c->lm_head, c->p_lg, rows, V, D, 0, true);
      if (rc) return rc;
      hipLaunchKernelGGL(k_ce_rows, dim3(rows), dim3(WG), 0, st, c->p_lg, targets + off + r0, c->p_ce + r0, V);
    }
    hipLaunchKernelGGL(k_loss_terms, dim3(1), dim3(WG), 0, st, c->p_ce, targets + off, T, V, c->d_rho + (size_t)b * L, L,
                       c->router, (size_t)L * D, lambda, alpha, terms_out + (size_t)b * 4);
    HIPCHK(c, hipGetLastError());
    off += T;
  }
  if (rho_out) HIPCHK(c, hipMemcpyAsync(rho_out, c->d_rho, (size_t)B * L * sizeof(float), hipMemcpyDeviceToDevice, st));
  HIPCHK(c, hipStreamSynchronize(st));
  release_sequences(c);          // a training pass leaves no sequence to decode
  return FIRST_OK;
}

int first_lora_merge(void* hip_stream, int32_t dtype, void* W, const float* A, const float* Bm, int32_t n, int32_t k, int32_t r,
                     float scale) {
  if (!W || !A || !Bm || n < 1 || k < 8 || k % 8 || r < 1 || r > LM_RMAX ||
      (dtype != FIRST_DTYPE_FP32 && dtype != FIRST_DTYPE_BF16)) {
    g_create_error = "first_lora_merge: null pointer, k not a multiple of 8, rank outside 1..32, or unknown dtype";
    return FIRST_ERR_ARG;
  }
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const int chunks = (k + LM_COLS - 1) / LM_COLS;
  const int want_y = std::max(1, (4 * device_cus() + chunks - 1) / chunks);          // about four workgroups per CU
  const int rows_per_wg = std::min(64, std::max(2 * LM_RG, ((n + want_y - 1) / want_y + 2 * LM_RG - 1) / (2 * LM_RG) * (2 * LM_RG)));
  const dim3 grid(chunks, (n + rows_per_wg - 1) / rows_per_wg);
  const size_t lds = ((size_t)r * LM_COLS + (size_t)rows_per_wg * r) * sizeof(float);
  hipError_t e;
  if (dtype == FIRST_DTYPE_BF16) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_lora_merge<bf16>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
      hipLaunchKernelGGL(k_lora_merge<bf16>, grid, dim3(WG), lds, st, reinterpret_cast<bf16*>(W), A, Bm, n, k, r, scale, rows_per_wg);
  } else {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_lora_merge<float>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess)
      hipLaunchKernelGGL(k_lora_merge<float>, grid, dim3(WG), lds, st, reinterpret_cast<float*>(W), A, Bm, n, k, r, scale, rows_per_wg);
  }
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) {
    g_create_error = std::string("first_lora_merge: ") + hipGetErrorString(e);
    return FIRST_ERR_HIP;
  }
  return FIRST_OK;
}

int first_op_gemv(void* hip_stream, int32_t dtype, const void* W, const float* x, float* y, int32_t n, int32_t k,
                  int32_t accumulate) {
  if (!W || !x || !y || n < 1 || k < 8 || k % 8 || (size_t)k * sizeof(float) > 60 * 1024 ||
      (dtype != FIRST_DTYPE_FP32 && dtype != FIRST_DTYPE_BF16))
    return fail(nullptr, FIRST_ERR_ARG, "first_op_gemv: bad argument");
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const int grid = gemv_grid(n, 4, device_cus());
  const size_t lds = ((size_t)k + WAVES) * sizeof(float);
  if (dtype == FIRST_DTYPE_BF16)
    hipLaunchKernelGGL(k_gemv<bf16>, dim3(grid), dim3(WG), lds, st, reinterpret_cast<const bf16*>(W), x, y, n, k, accumulate);
  else
    hipLaunchKernelGGL(k_gemv<float>, dim3(grid), dim3(WG), lds, st, reinterpret_cast<const float*>(W), x, y, n, k, accumulate);
  HIPCHK(nullptr, hipGetLastError());
  return FIRST_OK;
}

int first_step_timing(first_ctx* c, uint64_t* stamps, int32_t capacity, int32_t* n_out) {
  if (!c) return FIRST_ERR_ARG;
  if (!stamps || !n_out) return fail(c, FIRST_ERR_ARG, "first_step_timing: null output");
  if (c->B < 1) return fail(c, FIRST_ERR_STATE, "first_step_timing: no live sequence");
  int nk = 0;
  for (int i = 0; i < c->d.n_layers; ++i) nk += c->hmask[0][i] ? 1 : 0;
  const int n = (4 * nk + 1) * SK_TSLOTS;
  if (capacity < n) return fail(c, FIRST_ERR_ARG, "first_step_timing: buffer too small");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(stamps, c->d_tdbg, (size_t)n * sizeof(uint64_t), hipMemcpyDeviceToHost));
  *n_out = n;
  return FIRST_OK;
}


int first_op_gateup(first_ctx* c, int32_t layer, int32_t seq) {
  if (!c) return FIRST_ERR_ARG;
  if (layer < 0 || layer >= c->d.n_layers || seq < 0 || seq >= c->d.max_batch)
    return fail(c, FIRST_ERR_ARG, "first_op_gateup: layer or sequence out of range");
  DecParams p = base_params(c, seq, 1);
  set_layer(c, p, layer);
  const int grid = gemv_grid(2 * c->d.d_ffn, 4, c->num_cu);
  const size_t lds = ((size_t)c->d.d_model + WAVES) * sizeof(float);
  if (c->d.dtype == FIRST_DTYPE_BF16) hipLaunchKernelGGL(k_gateup<bf16>, dim3(grid), dim3(WG), lds, c->stream, p);
  else hipLaunchKernelGGL(k_gateup<float>, dim3(grid), dim3(WG), lds, c->stream, p);
  HIPCHK(c, hipGetLastError());
  return FIRST_OK;
}

int first_op_gemm_nt(void* hip_stream, int32_t dtype, const void* A, const void* W, float* C, int32_t m, int32_t n,
                     int32_t k, int32_t accumulate) {
  if (!A || !W || !C || m < 1 || n < 1 || k < 8 || k % 8 || (dtype != FIRST_DTYPE_FP32 && dtype != FIRST_DTYPE_BF16))
    return fail(nullptr, FIRST_ERR_ARG, "first_op_gemm_nt: bad argument");
  return launch_gemm(nullptr, reinterpret_cast<hipStream_t>(hip_stream), dtype, A, W, C, m, n, k, accumulate);
}

int first_op_gemm_nt_f32a(void* hip_stream, const float* A, const void* W, float* C, int32_t m, int32_t n, int32_t k,
                          int32_t accumulate) {
  if (!A || !W || !C || m < 1 || n < 1 || k < 8 || k % 8)
    return fail(nullptr, FIRST_ERR_ARG, "first_op_gemm_nt_f32a: bad argument");
  return launch_gemm(nullptr, reinterpret_cast<hipStream_t>(hip_stream), FIRST_DTYPE_BF16, A, W, C, m, n, k, accumulate, true);
}

}  // extern "C"
