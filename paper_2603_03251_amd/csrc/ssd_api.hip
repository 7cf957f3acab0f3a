// C ABI and round driver: owns device buffers, validates arguments, enqueues the kernels of one
// pre-speculation round (glue extend -> fan-out -> K branch-decode steps writing the speculation cache in place).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include <stdlib.h>

#include "common.h"
#include "fused.h"

namespace ssd {

static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}

namespace {

size_t elem_size(int dtype) { return dtype == SSD_BF16 ? 2 : 4; }

// Device allocations of one object, freed together.
struct Arena {
  std::vector<void*> ptrs;
  int alloc(void** out, size_t bytes) {
    *out = nullptr;
    if (bytes == 0) bytes = 16;
    hipError_t e = hipMalloc(out, bytes);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      set_error("hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
      return SSD_ENOMEM;
    }
    ptrs.push_back(*out);
    return SSD_OK;
  }
  void release() {
    for (void* p : ptrs) (void)hipFree(p);
    ptrs.clear();
  }
  void release_one(void* p) {
    for (size_t i = 0; i < ptrs.size(); ++i)
      if (ptrs[i] == p) {
        (void)hipFree(p);
        ptrs.erase(ptrs.begin() + (long)i);
        return;
      }
  }
};

__global__ void gather_chunk_tokens_kernel(int32_t* out, const int32_t* tokens, int stride, int B, int T, int start) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * T) return;
  int b = idx / T, t = idx % T;
  int src = start + t;
  out[idx] = src < stride ? tokens[(int64_t)b * stride + src] : 0;
}

}  // namespace
}  // namespace ssd

using namespace ssd;

struct ssd_model {
  Dims dims;
  int tie;
  Arena arena;
  void* embed = nullptr;       // row-major [V][d]
  void* lm_head = nullptr;     // GEMM layout (bf16: tile order)
  void* final_norm = nullptr;
  struct Layer {
    void *attn_norm, *wqkv, *wo, *mlp_norm, *w_gate, *w_up, *w_down;
  };
  std::vector<Layer> layers;
  // stream-order copies for the fused pass (bf16 models whose shape it supports)
  bool fused_ok = false;
  bool wide_ok = false;        // the wide pass (more than kFusedMaxRows rows) takes this shape too
  struct FusedW {
    FusedGemm qkv, o, gu, down;
  };
  std::vector<FusedW> fused_layers;
  FusedGemm fused_lm{};
  // the per-operator kernels' copies of the linear layers (tile order) can be given up: ssd_model_release_operator_weights
  bool operator_weights = true;
  mutable std::atomic<int> operator_contexts{0};   // live contexts that run the per-operator kernels
};

struct ssd_ctx {
  const ssd_model* model;
  int B, K, F, max_trunk;          // F: the largest fan-out of any accept length
  FanTable fan;                    // cache shape: accept length k owns rows fan.off[k] .. fan.off[k+1]-1 of a sequence
  int rows_per_seq;                // fan.off[K+1]
  int M;        // branch rows B (K+1) F
  int max_rows; // rows of the largest batched pass
  Arena arena;
  int trunk_ub = 0;   // host upper bound of every trunk_len[b]; 0 = trunk not loaded
  bool have_cache = false;
  // state
  int32_t* trunk_len;
  std::vector<void*> trunk_k, trunk_v;   // per layer [B][max_trunk][Hkv][D]
  std::vector<void*> suffix_k, suffix_v; // per layer [M][K][Hkv][D]
  // speculation cache
  int32_t* keys;
  int32_t* tokens;
  float* logits;
  float* hidden;
  float* glue_logits;
  float* glue_hidden;
  // scratch of a batched pass
  RowDesc* rows;
  float* cos_sin;
  int32_t* step_tokens;
  int32_t* exclude;
  float* h;          // residual stream, fp32
  float* qkv;        // fp32
  float* q;          // fp32
  // activations that feed a GEMM: fp32 (fp32 models) or bf16 head/remainder planes (bf16 models), 4 bytes/element
  void* xn;
  void* attn_out;
  void* act;
  float* attn_partial;
  void* sample_scratch = nullptr;   // per-row partial winners of the multi-block sampler
  void* top_f_scratch = nullptr;    // per-row, per-part candidates of the multi-block top-F
  float saguaro_c = 1.0f;           // downweighting constant of the sampling scheme sigma_{F,C}; 1 = off
  int32_t* sigma_ids = nullptr;     // [M][F] top-F of the current step's logits (saguaro_c < 1 only)
  int64_t attn_partial_floats = 0;
  // fused pass (see fused.h): 0 = per-operator kernels, 1 = one launch per phase, 2 = one persistent launch
  // paged trunk (App. B: block tables, pages of rejected tokens rolled back): the trunk of every layer is a pool of
  // 32-position pages shared by the sequences; a sequence's block j is page page_table[b][j]; page 0 is never handed out
  int kv_pages = 0;                      // pages of the pool, page 0 included; 0 = contiguous trunk per sequence
  int page_stride = 0;                   // blocks per sequence the table has room for
  int32_t* page_table_dev = nullptr;     // [B][page_stride]
  int32_t* page_table_host = nullptr;    // pinned mirror, the host's truth
  std::vector<int32_t> free_pages;       // stack of free page numbers
  std::vector<int> blocks_of;            // blocks a sequence holds pages for
  std::vector<int> ub_of;                // host upper bound of trunk_len per sequence (trunk_ub = their maximum)
  int fused_mode = 0;
  bool fused_wide = false;     // passes of up to kFusedWideRows rows through the wide kernel
  int fused_cap = 0;           // rows of one pass: kFusedMaxRows or kFusedWideRows
  int vt_stride = 0;
  FusedParams fp{};            // everything that does not change between passes
  FusedLayer* fused_layers_dev = nullptr;
  std::vector<FusedLayer> fused_layers_host;   // the same tables in host memory (wide passes launch phase by phase)
  unsigned* fused_bar = nullptr;
  unsigned* fused_err = nullptr;         // host-pinned word the kernel sets when a bounded wait expires
  hipEvent_t fused_done = nullptr;       // recorded behind every persistent launch of this context
  int flags = 0;
  int64_t fused_sync_words = 0; // barrier words, zeroed once (the barrier's epoch carries over from launch to launch)
  int64_t part_entries = 0;    // per-layer capacity of the attention partial buffers, in query rows
  int part_ns_max = 1;         // key splits they were sized for
  unsigned long long* phase_clocks = nullptr;
  const int32_t* forced_keys = nullptr;
  const int32_t* forced_tokens = nullptr;
  // optional per-segment timing of a round: K+3 events (start, glue, fan-out, K steps)
  std::vector<hipEvent_t> events;
  std::vector<hipEvent_t> kernel_events;   // fused contexts: start/end of the fused kernel of each branch-decode step
  bool timing = false;
};

namespace {

// Weight of a linear layer into the layout the GEMM streams: bf16 -> tile order, fp32 -> row-major copy.
int put_linear(int dtype, const void* src, void* dst, int N, int Kd, hipStream_t s) {
  if (dtype == SSD_BF16) return launch_tile_weights_bf16((const bf16_t*)src, (bf16_t*)dst, N, Kd, s);
  SSD_HIP(hipMemcpyAsync(dst, src, (size_t)N * Kd * 4, hipMemcpyDeviceToDevice, s));
  return SSD_OK;
}

// One layer's weights as the caller (or the on-device generator) holds them: row-major [out][in], model dtype.
struct LayerSrc {
  const void *attn_norm, *wq, *wk, *wv, *wo, *mlp_norm, *w_gate, *w_up, *w_down;
};

// A matrix into the stream order of the fused pass.  ks_wanted > 1: split the reduction dimension so that every
// workgroup of the grid gets a unit, if the shape allows.
int make_stream_order(ssd_model* m, int grid, FusedGemm* g, const void* s0, int r0, const void* s1, int r1, const void* s2, int r2,
                      int mode, int at, int ks_wanted, int Kd, hipStream_t s) {
  const int N = mode == 0 ? r0 + r1 + r2 : 2 * r0;
  const int NT = (N + 15) / 16, groups = (NT + at - 1) / at;
  int ks = 1;
  for (int k = ks_wanted; k > 1; k /= 2)
    if (groups * k <= grid && (Kd / 256) % (2 * k) == 0) { ks = k; break; }
  void* dst = nullptr;
  SSD_TRY(m->arena.alloc(&dst, (size_t)stream_order_elems(N, Kd, at) * 2));
  SSD_TRY(launch_retile_stream((const bf16_t*)s0, r0, (const bf16_t*)s1, r1, (const bf16_t*)s2, r2, mode, at, ks, Kd,
                               (bf16_t*)dst, s));
  // the fused passes multiply in fp16: convert in place (elementwise, same layout)
  SSD_TRY(launch_bf16_to_f16((const bf16_t*)dst, (bf16_t*)dst, stream_order_elems(N, Kd, at), s));
  g->w = (const bf16_t*)dst;
  g->KS = ks;
  g->KTW = Kd / 32 / kFusedWaves / ks;
  g->NT = NT;
  g->n_units = groups * ks;
  return SSD_OK;
}

// Model building in pieces, so that the source of a layer's weights may be a buffer that is reused for the next layer:
// build_begin, build_head, build_layer x n_layers, build_end, all on one stream.
int build_begin(ssd_model* m, int* grid) {
  const Dims& d = m->dims;
  m->layers.resize(d.n_layers);
  m->fused_ok = fused_supported(d, 1);
  *grid = 0;
  if (m->fused_ok) {
    SSD_TRY(fused_grid_size(grid));
    m->fused_layers.resize(d.n_layers);
  }
  return SSD_OK;
}

int build_head(ssd_model* m, int grid, const void* embed, const void* lm_head, const void* final_norm, hipStream_t s) {
  const Dims& d = m->dims;
  const size_t es = elem_size(d.dtype);
  SSD_TRY(m->arena.alloc(&m->embed, (size_t)d.vocab * d.d_model * es));
  SSD_HIP(hipMemcpyAsync(m->embed, embed, (size_t)d.vocab * d.d_model * es, hipMemcpyDeviceToDevice, s));
  SSD_TRY(m->arena.alloc(&m->final_norm, (size_t)d.d_model * es));
  SSD_HIP(hipMemcpyAsync(m->final_norm, final_norm, (size_t)d.d_model * es, hipMemcpyDeviceToDevice, s));
  const void* head_src = m->tie ? embed : lm_head;
  if (d.dtype == SSD_F32 && m->tie) m->lm_head = m->embed;
  else {
    SSD_TRY(m->arena.alloc(&m->lm_head, (size_t)d.vocab * d.d_model * es));
    SSD_TRY(put_linear(d.dtype, head_src, m->lm_head, d.vocab, d.d_model, s));
  }
  if (m->fused_ok)
    SSD_TRY(make_stream_order(m, grid, &m->fused_lm, head_src, d.vocab, nullptr, 0, nullptr, 0, 0, kAtLm, 1, d.d_model, s));
  return SSD_OK;
}

int build_layer(ssd_model* m, int grid, int l, const LayerSrc& w, hipStream_t s) {
  const Dims& d = m->dims;
  const size_t es = elem_size(d.dtype);
  const int qd = d.q_dim(), kvd = d.kv_dim();
  ssd_model::Layer& L = m->layers[l];
  SSD_TRY(m->arena.alloc(&L.attn_norm, (size_t)d.d_model * es));
  SSD_TRY(m->arena.alloc(&L.mlp_norm, (size_t)d.d_model * es));
  SSD_HIP(hipMemcpyAsync(L.attn_norm, w.attn_norm, (size_t)d.d_model * es, hipMemcpyDeviceToDevice, s));
  SSD_HIP(hipMemcpyAsync(L.mlp_norm, w.mlp_norm, (size_t)d.d_model * es, hipMemcpyDeviceToDevice, s));
  SSD_TRY(m->arena.alloc(&L.wqkv, (size_t)d.qkv_dim() * d.d_model * es));
  char* qkv = (char*)L.wqkv;
  SSD_TRY(put_linear(d.dtype, w.wq, qkv, qd, d.d_model, s));
  SSD_TRY(put_linear(d.dtype, w.wk, qkv + (size_t)qd * d.d_model * es, kvd, d.d_model, s));
  SSD_TRY(put_linear(d.dtype, w.wv, qkv + (size_t)(qd + kvd) * d.d_model * es, kvd, d.d_model, s));
  SSD_TRY(m->arena.alloc(&L.wo, (size_t)d.d_model * qd * es));
  SSD_TRY(put_linear(d.dtype, w.wo, L.wo, d.d_model, qd, s));
  SSD_TRY(m->arena.alloc(&L.w_gate, (size_t)d.d_ffn * d.d_model * es));
  SSD_TRY(put_linear(d.dtype, w.w_gate, L.w_gate, d.d_ffn, d.d_model, s));
  SSD_TRY(m->arena.alloc(&L.w_up, (size_t)d.d_ffn * d.d_model * es));
  SSD_TRY(put_linear(d.dtype, w.w_up, L.w_up, d.d_ffn, d.d_model, s));
  SSD_TRY(m->arena.alloc(&L.w_down, (size_t)d.d_model * d.d_ffn * es));
  SSD_TRY(put_linear(d.dtype, w.w_down, L.w_down, d.d_model, d.d_ffn, s));
  if (m->fused_ok) {
    ssd_model::FusedW& F = m->fused_layers[l];
    SSD_TRY(make_stream_order(m, grid, &F.qkv, w.wq, qd, w.wk, kvd, w.wv, kvd, 0, kAtQkv, 1, d.d_model, s));
    SSD_TRY(make_stream_order(m, grid, &F.o, w.wo, d.d_model, nullptr, 0, nullptr, 0, 0, kAtO, 2, qd, s));
    SSD_TRY(make_stream_order(m, grid, &F.gu, w.w_gate, d.d_ffn, w.w_up, d.d_ffn, nullptr, 0, 1, kAtGu, 1, d.d_model, s));
    SSD_TRY(make_stream_order(m, grid, &F.down, w.w_down, d.d_model, nullptr, 0, nullptr, 0, 0, kAtDown, 4, d.d_ffn, s));
  }
  return SSD_OK;
}

int build_end(ssd_model* m, int grid) {
  if (!m->fused_ok) return SSD_OK;
  // the layer phases of the narrow pass give every workgroup at most one unit and unroll over the k-tiles of a wavefront
  auto fits = [&](const FusedGemm& g, int max_ktw) {
    return g.n_units <= grid && (g.KTW == 2 || g.KTW == 4 || g.KTW == 8) && g.KTW <= max_ktw;
  };
  m->wide_ok = fused_wide_gemm_ok(m->fused_lm, kAtLm);
  for (const ssd_model::FusedW& F : m->fused_layers) {
    if (!fits(F.qkv, 8) || !fits(F.o, 8) || !fits(F.down, 8)) m->fused_ok = false;
    if (!fused_wide_gemm_ok(F.qkv, kAtQkv) || !fused_wide_gemm_ok(F.o, kAtO) || !fused_wide_gemm_ok(F.gu, kAtGu) ||
        !fused_wide_gemm_ok(F.down, kAtDown))
      m->wide_ok = false;
  }
  m->wide_ok = m->wide_ok && m->fused_ok;
  return SSD_OK;
}

int build_model(ssd_model* m, const ssd_model_weights* w, hipStream_t s) {
  int grid = 0;
  SSD_TRY(build_begin(m, &grid));
  SSD_TRY(build_head(m, grid, w->d_embed, w->d_lm_head, w->d_final_norm, s));
  for (int l = 0; l < m->dims.n_layers; ++l) {
    const LayerSrc src = {w->h_attn_norm[l], w->h_wq[l], w->h_wk[l], w->h_wv[l], w->h_wo[l], w->h_mlp_norm[l],
                          w->h_w_gate[l], w->h_w_up[l], w->h_w_down[l]};
    SSD_TRY(build_layer(m, grid, l, src, s));
  }
  return build_end(m, grid);
}

// Random-init weights generated on the device, layer by layer through one set of scratch matrices (every matrix
// N(0, std)-like from the integer hash of kernels_init.hip, every RMSNorm gain 1).
int build_model_random(ssd_model* m, uint64_t seed, double std, hipStream_t s) {
  const Dims& d = m->dims;
  const size_t es = elem_size(d.dtype);
  const int64_t qd = d.q_dim(), kvd = d.kv_dim(), dm = d.d_model, ff = d.d_ffn, V = d.vocab;
  Arena tmp;
  int grid = 0;
  int st = build_begin(m, &grid);
  void *embed = nullptr, *head = nullptr, *ones = nullptr, *wq = nullptr, *wk = nullptr, *wv = nullptr, *wo = nullptr, *wg = nullptr,
       *wu = nullptr, *wd = nullptr;
  auto A = [&](void** q, size_t bytes) { if (st == SSD_OK) st = tmp.alloc(q, bytes); };
  auto T = [&](int r) { if (st == SSD_OK) st = r; };
  A(&embed, (size_t)V * dm * es);
  if (!m->tie) A(&head, (size_t)V * dm * es);
  A(&ones, (size_t)dm * es);
  if (st == SSD_OK) {
    T(launch_fill_hashed(d.dtype, embed, V * dm, seed, 0, std, s));
    if (!m->tie) T(launch_fill_hashed(d.dtype, head, V * dm, seed, 1, std, s));
    T(launch_fill_const(d.dtype, ones, dm, 1.0f, s));
    if (st == SSD_OK) st = build_head(m, grid, embed, head, ones, s);
  }
  A(&wq, (size_t)qd * dm * es); A(&wk, (size_t)kvd * dm * es); A(&wv, (size_t)kvd * dm * es); A(&wo, (size_t)dm * qd * es);
  A(&wg, (size_t)ff * dm * es); A(&wu, (size_t)ff * dm * es); A(&wd, (size_t)dm * ff * es);
  for (int l = 0; l < d.n_layers && st == SSD_OK; ++l) {
    const uint64_t id = 16 + 16 * (uint64_t)l;
    T(launch_fill_hashed(d.dtype, wq, qd * dm, seed, id + 0, std, s));
    T(launch_fill_hashed(d.dtype, wk, kvd * dm, seed, id + 1, std, s));
    T(launch_fill_hashed(d.dtype, wv, kvd * dm, seed, id + 2, std, s));
    T(launch_fill_hashed(d.dtype, wo, dm * qd, seed, id + 3, std, s));
    T(launch_fill_hashed(d.dtype, wg, ff * dm, seed, id + 4, std, s));
    T(launch_fill_hashed(d.dtype, wu, ff * dm, seed, id + 5, std, s));
    T(launch_fill_hashed(d.dtype, wd, dm * ff, seed, id + 6, std, s));
    const LayerSrc src = {ones, wq, wk, wv, wo, ones, wg, wu, wd};
    if (st == SSD_OK) st = build_layer(m, grid, l, src, s);   // same stream: the next layer's fill follows this layer's re-tiling
  }
  if (st == SSD_OK) st = build_end(m, grid);
  hipError_t e = hipStreamSynchronize(s);
  tmp.release();
  if (st == SSD_OK && e != hipSuccess) { set_error("hipStreamSynchronize failed: %s", hipGetErrorString(e)); st = SSD_EHIP; }
  return st;
}

// Persistent launches spin on grid barriers, so every workgroup of one must be resident at once: two of them running
// side by side (two contexts, or one context driven from two streams) could each hold part of the compute units and
// wait for the rest for ever.  Every persistent launch therefore waits, on the device, for the previous one of the
// process wherever that ran on another stream.
std::mutex g_fused_mu;
hipEvent_t g_fused_last_event = nullptr;
hipStream_t g_fused_last_stream = nullptr;
const ssd_ctx* g_fused_last_ctx = nullptr;

// Once a bounded wait of the fused pass has expired the context's barrier state and everything computed since are
// invalid: every later call fails until ssd_ctx_recover.  The word lives in pinned host memory, so this costs one load.
int ctx_fault(const ssd_ctx* c, const char* who) {
  if (c->fused_mode && c->fused_err && *(volatile const unsigned*)c->fused_err) {
    set_error("%s: a bounded wait inside the fused pass expired on this context (were the compute units shared with another "
              "persistent kernel?); results since then are invalid, call ssd_ctx_recover", who);
    return SSD_EHIP;
  }
  return SSD_OK;
}

// Pages for positions 0 .. positions-1 of sequence b (paged contexts; no-op otherwise).  New entries go to the host
// mirror; *dirty tells the caller to upload the table before the next kernel.
int pages_ensure(ssd_ctx* c, int b, int positions, bool* dirty) {
  if (!c->kv_pages) return SSD_OK;
  const int need = (positions + 31) / 32;
  if (need > c->page_stride) { set_error("sequence %d: %d positions exceed the page table", b, positions); return SSD_ESTATE; }
  while (c->blocks_of[b] < need) {
    if (c->free_pages.empty()) {
      set_error("out of KV pages (%d in the pool): sequence %d needs block %d; release a sequence or tighten the bounds "
                "(ssd_ctx_refresh_bounds)", c->kv_pages, b, c->blocks_of[b]);
      return SSD_ENOMEM;
    }
    c->page_table_host[(size_t)b * c->page_stride + c->blocks_of[b]++] = c->free_pages.back();
    c->free_pages.pop_back();
    *dirty = true;
  }
  return SSD_OK;
}

// Page rollback: sequence b keeps the pages of its first `positions` positions, the rest go back to the pool.  The
// caller has synchronised the streams that may still read them.
void pages_release_beyond(ssd_ctx* c, int b, int positions, bool* dirty) {
  if (!c->kv_pages) return;
  const int keep = (positions + 31) / 32;
  while (c->blocks_of[b] > keep) {
    int32_t& e = c->page_table_host[(size_t)b * c->page_stride + --c->blocks_of[b]];
    c->free_pages.push_back(e);
    e = 0;
    *dirty = true;
  }
}

int pages_upload(ssd_ctx* c, hipStream_t s) {
  SSD_HIP(hipMemcpyAsync(c->page_table_dev, c->page_table_host, sizeof(int32_t) * (size_t)c->B * c->page_stride,
                         hipMemcpyHostToDevice, s));
  return SSD_OK;
}

// Before a pass that writes trunk positions up to (bound of sequence b) + extra of sequences [b0, b0 + nb)
int pages_for_pass(ssd_ctx* c, int b0, int nb, int extra, hipStream_t s) {
  if (!c->kv_pages) return SSD_OK;
  bool dirty = false;
  for (int b = b0; b < b0 + nb; ++b) SSD_TRY(pages_ensure(c, b, c->ub_of[b] + extra, &dirty));
  return dirty ? pages_upload(c, s) : SSD_OK;
}

void set_bounds(ssd_ctx* c, const int32_t* lens) {
  c->trunk_ub = 0;
  for (int b = 0; b < c->B; ++b) {
    c->ub_of[b] = lens[b];
    c->trunk_ub = lens[b] > c->trunk_ub ? lens[b] : c->trunk_ub;
  }
}

// The same pass through the fused kernel: attention work split for this pass's shape, then one launch per group of
// whole sequences that fits kFusedMaxRows rows (one launch for the few-row workloads the kernel is built for; a batch
// with more rows streams the weights once per group).
// seq_base: the pass's rows belong to sequences seq_base, seq_base + 1, .. (rows, tokens and outputs are indexed from 0)
int fused_forward(ssd_ctx* c, int M, const int32_t* tokens, int rows_per_seq, int max_vis, int branch_depth, float* logits,
                  int64_t logits_ld, float* hidden, int64_t hidden_ld, int seq_base, hipStream_t s) {
  FusedParams p = c->fp;
  p.R = rows_per_seq;
  p.is_branch = branch_depth >= 0;
  p.suffix_len = branch_depth >= 0 ? branch_depth + 1 : 0;
  p.tv_ub = max_vis > 0 ? max_vis : 0;
  const int RG = p.R * p.G;
  p.QT = (RG + 15) / 16;
  p.SL = c->K + 1 <= 8 ? 8 : 16;
  const int p_ub = max_vis > 1 ? max_vis : 1;
  const int n_seq = M / rows_per_seq;
  const int per_pass = c->fused_cap / rows_per_seq;
  // Key splits of the stored trunk: the attention phase lasts (rounds of units over the grid) x (a unit's 32-key blocks
  // per wavefront + its fixed part), and more than one split adds a merge (a phase of its own in wide passes, the last
  // unit of a tile to arrive in narrow ones).  Costs in microseconds as measured
  // on the 1B shape; the choice only affects speed.
  {
    const int seqs = n_seq < per_pass ? n_seq : (per_pass > 0 ? per_pass : 1);
    const int pairs = seqs * p.Hkv * (c->fused_wide ? (p.QT + kFusedWideQueryTiles - 1) / kFusedWideQueryTiles : p.QT);
    int best = 1;
    float best_cost = 0.f;
    const int ns_cap = c->part_ns_max;                     // what the partial-softmax buffers were sized for
    const float merge_cost = c->fused_wide ? 5.0f : 4.0f;  // a phase of its own / the last unit of a tile to arrive (its arrival
                                                           // count and the other splits' partial results each cost a memory round trip)
    for (int ns = 1; ns <= ns_cap && ns <= 16; ++ns) {
      const int keys = (p_ub + ns - 1) / ns;
      const int blocks = ((keys + 31) / 32 + kFusedWaves - 1) / kFusedWaves;
      const int rounds = (pairs * ns + p.nwg - 1) / p.nwg;
      const float cost = rounds * (0.9f * blocks + 3.0f) + (ns > 1 ? merge_cost : 0.f);
      if (ns == 1 || cost < best_cost) { best = ns; best_cost = cost; }
    }
    p.KPU = ((p_ub + best - 1) / best + 31) / 32 * 32;
    p.NS = (p_ub + p.KPU - 1) / p.KPU;
  }
  if (per_pass < 1 || n_seq * rows_per_seq != M) {
    set_error("fused pass: %d rows of %d per sequence do not fit passes of %d rows", M, rows_per_seq, c->fused_cap);
    return SSD_ESTATE;
  }
  const int last = (logits || hidden) ? fused_last_phase(p.L) : fused_last_phase(p.L) - 1;
  const bool timed = c->timing && branch_depth >= 0 && 2 * branch_depth + 1 < (int)c->kernel_events.size();
  const bool persistent = c->fused_mode == 2;
  std::unique_lock<std::mutex> serial(g_fused_mu, std::defer_lock);
  if (persistent) {
    serial.lock();
    if (g_fused_last_event && g_fused_last_stream != s) SSD_HIP(hipStreamWaitEvent(s, g_fused_last_event, 0));
  }
  if (timed) SSD_HIP(hipEventRecord(c->kernel_events[2 * branch_depth], s));
  for (int s0 = 0; s0 < n_seq; s0 += per_pass) {
    const int nb = n_seq - s0 < per_pass ? n_seq - s0 : per_pass;
    const int64_t row0 = (int64_t)s0 * rows_per_seq;
    p.B = nb;
    p.M = nb * rows_per_seq;
    p.layers = c->fused_layers_dev + (size_t)(seq_base + s0) * p.L;
    p.pages = c->kv_pages ? c->page_table_dev + (size_t)(seq_base + s0) * c->page_stride : nullptr;
    p.page_stride = c->page_stride;
    p.rows = c->rows + row0;
    p.cos_sin = c->cos_sin + row0 * (c->model->dims.head_dim / 2) * 2;
    p.tokens = tokens + row0;
    p.logits = logits ? logits + row0 * logits_ld : nullptr;
    p.logits_ld = logits_ld;
    p.hidden = hidden ? hidden + row0 * hidden_ld : nullptr;
    p.hidden_ld = hidden_ld;
    p.n_attn_units = p.B * p.Hkv * (c->fused_wide ? (p.QT + kFusedWideQueryTiles - 1) / kFusedWideQueryTiles : p.QT) * p.NS;
    p.n_pair_units = (p.M * p.Hq + kFusedWaves - 1) / kFusedWaves;
    if (p.NS > 1 && (int64_t)p.B * p.Hkv * p.NS * p.QT * 16 > c->part_entries) {
      set_error("fused pass: attention partial buffer too small (%d splits, %d query tiles)", p.NS, p.QT);
      return SSD_ESTATE;
    }
    if (c->fused_wide) SSD_TRY(launch_fused_wide(p, c->fused_layers_host.data() + (size_t)(seq_base + s0) * p.L, 0, last, s));
    else SSD_TRY(launch_fused(p, 0, last, persistent, s));
  }
  if (timed) SSD_HIP(hipEventRecord(c->kernel_events[2 * branch_depth + 1], s));
  if (persistent) {
    SSD_HIP(hipEventRecord(c->fused_done, s));
    g_fused_last_event = c->fused_done;
    g_fused_last_stream = s;
    g_fused_last_ctx = c;
  }
  return SSD_OK;
}

// One batched pass of the decoder over `M` rows whose descriptors and rotary tables are already in ctx->rows /
// ctx->cos_sin.  Logits (fp32, row stride logits_ld) and final-norm hidden states are optional.
// max_vis: host bound of the stored trunk positions any row sees; branch_depth: decode step of branch rows, -1 for an extend.
int forward_rows(ssd_ctx* c, int M, const int32_t* tokens, int rows_per_seq, int max_vis, int branch_depth, float* logits,
                 int64_t logits_ld, float* hidden, int64_t hidden_ld, int seq_base, hipStream_t s) {
  const ssd_model* m = c->model;
  const Dims& d = m->dims;
  if (c->fused_mode)
    return fused_forward(c, M, tokens, rows_per_seq, max_vis, branch_depth, logits, logits_ld, hidden, hidden_ld, seq_base, s);
  const int dt = d.dtype;
  const int64_t R = c->max_rows;     // plane stride of an activation buffer = R * columns
  SSD_TRY(launch_embed(dt, m->embed, tokens, c->h, M, d.d_model, d.vocab, s));
  for (int l = 0; l < d.n_layers; ++l) {
    const ssd_model::Layer& L = m->layers[l];
    SSD_TRY(launch_rmsnorm(dt, c->h, L.attn_norm, c->xn, R * d.d_model, nullptr, 0, M, d.d_model, d.rms_eps, s));
    SSD_TRY(launch_gemm(dt, EPI_STORE_F32, c->xn, R * d.d_model, L.wqkv, nullptr, c->qkv, d.qkv_dim(), 0, M, d.qkv_dim(),
                        d.d_model, s));
    SSD_TRY(launch_rope_append(dt, c->qkv, c->rows, c->cos_sin, c->q, c->trunk_k[l], c->trunk_v[l], c->suffix_k[l],
                               c->suffix_v[l], M, d.n_q_heads, d.n_kv_heads, d.head_dim, c->max_trunk, c->K, s));
    AttnArgs a;
    a.q = c->q; a.trunk_k = c->trunk_k[l]; a.trunk_v = c->trunk_v[l]; a.suffix_k = c->suffix_k[l];
    a.suffix_v = c->suffix_v[l]; a.out = c->attn_out; a.out_plane = R * d.q_dim(); a.rows = c->rows; a.partial = c->attn_partial; a.partial_floats = c->attn_partial_floats; a.M = M;
    a.n_q_heads = d.n_q_heads; a.n_kv_heads = d.n_kv_heads; a.head_dim = d.head_dim; a.max_trunk = c->max_trunk;
    a.suffix_cap = c->K; a.rows_per_seq = rows_per_seq;
    // here the tokens of an extend are trunk positions too (they are appended before the attention runs)
    a.max_vis = max_vis + (branch_depth < 0 ? rows_per_seq : 0);
    SSD_TRY(launch_attention(dt, a, s));
    SSD_TRY(launch_gemm(dt, EPI_RESIDUAL_ADD, c->attn_out, R * d.q_dim(), L.wo, nullptr, c->h, d.d_model, 0, M, d.d_model,
                        d.q_dim(), s));
    SSD_TRY(launch_rmsnorm(dt, c->h, L.mlp_norm, c->xn, R * d.d_model, nullptr, 0, M, d.d_model, d.rms_eps, s));
    SSD_TRY(launch_gemm(dt, EPI_SWIGLU, c->xn, R * d.d_model, L.w_gate, L.w_up, c->act, d.d_ffn, R * d.d_ffn, M, d.d_ffn,
                        d.d_model, s));
    SSD_TRY(launch_gemm(dt, EPI_RESIDUAL_ADD, c->act, R * d.d_ffn, L.w_down, nullptr, c->h, d.d_model, 0, M, d.d_model,
                        d.d_ffn, s));
  }
  if (logits || hidden) {
    SSD_TRY(launch_rmsnorm(dt, c->h, m->final_norm, c->xn, R * d.d_model, hidden, hidden_ld, M, d.d_model, d.rms_eps, s));
    if (logits) SSD_TRY(launch_gemm(dt, EPI_STORE_F32, c->xn, R * d.d_model, m->lm_head, nullptr, logits, logits_ld, 0, M,
                                    d.vocab, d.d_model, s));
  }
  return SSD_OK;
}

// Extend of sequences [b0, b0 + nb): tokens [nb][T], outputs [nb][T][..]
int extend_rows(ssd_ctx* c, const int32_t* tokens, int T, int offset, float* logits, float* hidden, int b0, int nb, hipStream_t s) {
  const Dims& d = c->model->dims;
  SSD_TRY(pages_for_pass(c, b0, nb, offset + T, s));
  SSD_TRY(launch_setup_extend_rows(c->rows, c->cos_sin, c->trunk_len, nb, T, offset, d.head_dim / 2, d.rope_theta, b0, s));
  int ub = 0;
  for (int b = b0; b < b0 + nb; ++b) ub = c->ub_of[b] > ub ? c->ub_of[b] : ub;
  return forward_rows(c, nb * T, tokens, T, ub + offset, -1, logits, d.vocab, hidden, d.d_model, b0, s);
}

// Workspace and constant parameters of the fused pass.
int fused_setup(ssd_ctx* c) {
  const ssd_model* m = c->model;
  const Dims& d = m->dims;
  const int L = d.n_layers;
  FusedParams& p = c->fp;
  SSD_TRY(fused_grid_size(&p.nwg));
  p.L = L; p.d = d.d_model; p.qd = d.q_dim(); p.kvd = d.kv_dim(); p.qkvd = d.qkv_dim(); p.ffn = d.d_ffn; p.V = d.vocab;
  p.Hq = d.n_q_heads; p.Hkv = d.n_kv_heads; p.G = d.n_q_heads / d.n_kv_heads; p.eps = d.rms_eps;
  p.embed = (const bf16_t*)m->embed;
  p.final_norm = (const bf16_t*)m->final_norm;
  p.lm = m->fused_lm;
  p.B = c->B;
  p.rows = c->rows;
  p.cos_sin = c->cos_sin;
  p.max_trunk = c->max_trunk;
  p.vt_stride = c->vt_stride;
  p.suffix_cap = c->K;
  const size_t MPr = (size_t)c->fused_cap;
  const size_t nv = 2 * (size_t)L + 1;
  int st = SSD_OK;
  auto A = [&](void** q, size_t bytes) { if (st == SSD_OK) st = c->arena.alloc(q, bytes); };
  A((void**)&p.h, nv * MPr * p.d * 4);
  A((void**)&p.xn, nv * 2 * MPr * p.d * 2);
  A((void**)&p.ssq, nv * (p.d / 16) * MPr * 4);
  A((void**)&p.qkv, (size_t)L * MPr * p.qkvd * 4);
  A((void**)&p.att, (size_t)L * 2 * MPr * p.qd * 2);
  A((void**)&p.act, (size_t)L * 2 * MPr * p.ffn * 2);
  // attention partials (used only when the trunk is split over several units: more than 2048 visible keys)
  const int r_max = c->rows_per_seq > c->K + 1 ? c->rows_per_seq : c->K + 1;
  const int qt_max = (r_max * p.G + 15) / 16;
  // narrow passes split shorter trunks too (their units merge the splits themselves, at no barrier)
  const int ns_max = c->fused_wide ? (c->max_trunk + 2047) / 2048 + 1 : std::max((c->max_trunk + 2047) / 2048 + 1, 8);
  c->part_ns_max = ns_max;
  c->part_entries = (int64_t)p.B * p.Hkv * ns_max * qt_max * 16;
  p.part_layer_stride = c->part_entries;
  A((void**)&p.part_o, (size_t)L * c->part_entries * 64 * 4);
  A((void**)&p.part_ml, (size_t)L * c->part_entries * 2 * 4);
  p.arrivals_stride = (int64_t)p.B * p.Hkv * qt_max;
  A((void**)&p.arrivals, (size_t)L * p.arrivals_stride * 4);
  A((void**)&p.qkv_flags, (size_t)L * 128 * 4);
  // K-split scratch: per (layer, qkv / o / down) partial tiles.  A word of 0xffffffff means "not written in this
  // launch": filled once here, and the kernel's reader restores it after taking a tile.
  int64_t fix_tiles = 1;   // most (feature tile, slice) pairs of a K-split layer, padding tiles of the last unit included
  for (int l = 0; l < L; ++l)
    for (const auto& ga : {std::make_pair(&m->fused_layers[l].qkv, kAtQkv), std::make_pair(&m->fused_layers[l].o, kAtO),
                           std::make_pair(&m->fused_layers[l].down, kAtDown)})
      if (ga.first->KS > 1 && (int64_t)ga.first->n_units * ga.second > fix_tiles) fix_tiles = (int64_t)ga.first->n_units * ga.second;
  p.fix_stride = fix_tiles * (kFusedMaxRows / 16) * 256;   // x row tiles x 256 floats (narrow passes only)
  c->fused_sync_words = kFusedSyncWords;
  A((void**)&p.fix_buf, (size_t)L * 3 * p.fix_stride * 4);
  A((void**)&c->fused_bar, (size_t)(c->fused_sync_words + 64) * 4);
  A((void**)&c->fused_layers_dev, sizeof(FusedLayer) * L * c->B);
  SSD_TRY(st);
  // every workgroup of a persistent launch has to be resident at once
  // xn, att, act as one fp16 plane unless two planes are asked for; q, p as asked
  p.planes = ((c->flags >> 8) & 31) | (c->flags & SSD_CTX_TWO_PLANES ? 0 : 7);
  if (!c->fused_wide && !fused_planes_supported(p.planes)) { set_error("fused pass: plane configuration %d is not compiled in", p.planes); return SSD_EINVAL; }
  if (c->fused_mode == 2) SSD_TRY(fused_check_residency(p.nwg, p.planes, c->kv_pages ? 1 : 0));
  {
    void* host_word = nullptr;
    hipError_t e = hipHostMalloc(&host_word, 64, hipHostMallocMapped);
    if (e != hipSuccess) { (void)hipGetLastError(); set_error("hipHostMalloc failed: %s", hipGetErrorString(e)); return SSD_ENOMEM; }
    c->fused_err = (unsigned*)host_word;
    *c->fused_err = 0u;
  }
  SSD_HIP(hipEventCreateWithFlags(&c->fused_done, hipEventDisableTiming));
  p.bar = c->fused_bar;
  p.err = c->fused_err;
  p.spin_limit = kFusedSpinLimit;
  SSD_TRY(fused_init_barrier(c->fused_bar, 0u, p.nwg));
  SSD_TRY(fused_init_group_flags(p.qkv_flags, L, 0u));
  SSD_HIP(hipMemset(p.fix_buf, 0xff, (size_t)L * 3 * p.fix_stride * 4));
  SSD_HIP(hipMemset(p.arrivals, 0, (size_t)L * p.arrivals_stride * 4));
  // Group sync of the narrow persistent pass (no grid barrier between qkv and attention): the qkv units of a KV head's
  // group (2 G + 2 + 2 units of 32 features) go to workgroups of the XCD that head's attention units run on
  p.qkv_ug = 0;
  {
    const int ug = 2 * p.G + 4;
    bool fits = c->fused_mode == 2 && !c->fused_wide && p.Hkv <= 8 && 8 % p.Hkv == 0 && ug <= 16 && 8 * ug <= p.nwg;
    for (int l = 0; l < L && fits; ++l)
      fits = m->fused_layers[l].qkv.KS == 1 && m->fused_layers[l].qkv.n_units == 2 * p.Hq + 4 * p.Hkv;
    if (fits) p.qkv_ug = ug;
  }
  p.deep = 1;   // ring depth of the gate/up and LM-head streaming loops
  for (int l = 0; l < L; ++l)
    if (m->fused_layers[l].gu.KTW % 4) p.deep = 0;
  if (m->fused_lm.KTW % 4) p.deep = 0;
  // Layer tables, one per first sequence of a pass: a pass takes as many whole sequences as fit kFusedMaxRows rows, and
  // the kernel numbers sequences and rows from 0, so the KV pointers of table s start at sequence s (and at its first
  // branch row).
  std::vector<FusedLayer>& host = c->fused_layers_host;
  host.assign((size_t)L * c->B, FusedLayer{});
  const size_t kvd = (size_t)d.kv_dim();
  const size_t branch_rows = (size_t)c->rows_per_seq;
  for (int l = 0; l < L; ++l) {
    // masked keys still feed the value MFMA with weight 0: everything there must be finite
    const size_t trunk_elems = c->kv_pages ? (size_t)c->kv_pages * 32 * kvd : (size_t)c->B * kvd * c->vt_stride;
    SSD_HIP(hipMemset(c->trunk_k[l], 0, trunk_elems * 2));
    SSD_HIP(hipMemset(c->trunk_v[l], 0, trunk_elems * 2));
    for (int sq = 0; sq < c->B; ++sq) {
      FusedLayer& F = host[(size_t)sq * L + l];
      F.qkv = m->fused_layers[l].qkv; F.o = m->fused_layers[l].o; F.gu = m->fused_layers[l].gu; F.down = m->fused_layers[l].down;
      F.attn_norm = (const bf16_t*)m->layers[l].attn_norm;
      F.mlp_norm = (const bf16_t*)m->layers[l].mlp_norm;
      // paged: every sequence addresses the one pool through its row of the page table
      F.trunk_k = (bf16_t*)c->trunk_k[l] + (c->kv_pages ? 0 : (size_t)sq * kvd * c->vt_stride);
      F.trunk_vt = (bf16_t*)c->trunk_v[l] + (c->kv_pages ? 0 : (size_t)sq * kvd * c->vt_stride);
      F.suffix_k = (bf16_t*)c->suffix_k[l] + (size_t)sq * branch_rows * c->K * kvd;
      F.suffix_v = (bf16_t*)c->suffix_v[l] + (size_t)sq * branch_rows * c->K * kvd;
    }
  }
  SSD_HIP(hipMemcpy(c->fused_layers_dev, host.data(), sizeof(FusedLayer) * host.size(), hipMemcpyHostToDevice));
  p.layers = c->fused_layers_dev;
  return SSD_OK;
}

}  // namespace

extern "C" {

const char* ssd_last_error(void) { return g_error; }

static int check_model_config(const ssd_model_config* cfg) {
  SSD_CHECK_ARG(cfg->dtype == SSD_F32 || cfg->dtype == SSD_BF16, "dtype %d unknown", cfg->dtype);
  SSD_CHECK_ARG(cfg->n_layers >= 1 && cfg->d_model >= 1 && cfg->n_q_heads >= 1 && cfg->n_kv_heads >= 1 &&
                    cfg->d_ffn >= 1 && cfg->vocab >= 2,
                "model sizes must be positive (vocab >= 2)");
  SSD_CHECK_ARG(cfg->head_dim == 64 || cfg->head_dim == 128, "head_dim %d not supported (64 or 128)", cfg->head_dim);
  SSD_CHECK_ARG(cfg->n_q_heads % cfg->n_kv_heads == 0, "n_q_heads must be a multiple of n_kv_heads");
  SSD_CHECK_ARG(cfg->d_model % 4 == 0 && cfg->d_ffn % 4 == 0, "d_model and d_ffn must be multiples of 4");
  return SSD_OK;
}

static ssd_model* new_model(const ssd_model_config* cfg) {
  ssd_model* m = new (std::nothrow) ssd_model();
  if (!m) { set_error("out of host memory"); return nullptr; }
  m->dims.n_layers = cfg->n_layers; m->dims.d_model = cfg->d_model; m->dims.n_q_heads = cfg->n_q_heads;
  m->dims.n_kv_heads = cfg->n_kv_heads; m->dims.head_dim = cfg->head_dim; m->dims.d_ffn = cfg->d_ffn;
  m->dims.vocab = cfg->vocab; m->dims.dtype = cfg->dtype; m->dims.rope_theta = cfg->rope_theta;
  m->dims.rms_eps = cfg->rms_eps;
  m->tie = cfg->tie_embeddings ? 1 : 0;
  return m;
}

int ssd_model_create_random(const ssd_model_config* cfg, uint64_t seed, void* stream, ssd_model** out) {
  SSD_CHECK_ARG(cfg && out, "ssd_model_create_random: null argument");
  *out = nullptr;
  SSD_TRY(check_model_config(cfg));
  ssd_model* m = new_model(cfg);
  if (!m) return SSD_ENOMEM;
  int st = build_model_random(m, seed, 0.02, (hipStream_t)stream);
  if (st != SSD_OK) { m->arena.release(); delete m; return st; }
  *out = m;
  return SSD_OK;
}

int ssd_model_create(const ssd_model_config* cfg, const ssd_model_weights* w, void* stream, ssd_model** out) {
  SSD_CHECK_ARG(cfg && w && out, "ssd_model_create: null argument");
  *out = nullptr;
  SSD_TRY(check_model_config(cfg));
  SSD_CHECK_ARG(w->d_embed && w->d_final_norm && (cfg->tie_embeddings || w->d_lm_head), "null weight pointer");
  SSD_CHECK_ARG(w->h_attn_norm && w->h_wq && w->h_wk && w->h_wv && w->h_wo && w->h_mlp_norm && w->h_w_gate &&
                    w->h_w_up && w->h_w_down,
                "null per-layer pointer table");
  for (int l = 0; l < cfg->n_layers; ++l)
    SSD_CHECK_ARG(w->h_attn_norm[l] && w->h_wq[l] && w->h_wk[l] && w->h_wv[l] && w->h_wo[l] && w->h_mlp_norm[l] &&
                      w->h_w_gate[l] && w->h_w_up[l] && w->h_w_down[l],
                  "null weight pointer in layer %d", l);
  ssd_model* m = new_model(cfg);
  if (!m) return SSD_ENOMEM;
  int st = build_model(m, w, (hipStream_t)stream);
  if (st != SSD_OK) { m->arena.release(); delete m; return st; }
  *out = m;
  return SSD_OK;
}

int ssd_model_release_operator_weights(ssd_model* m) {
  SSD_CHECK_ARG(m, "ssd_model_release_operator_weights: null model");
  if (!m->operator_weights) return SSD_OK;
  if (!m->fused_ok) { set_error("this model's shape is served by the per-operator kernels only: their weights stay"); return SSD_ESTATE; }
  if (m->operator_contexts.load() > 0) {
    set_error("%d context(s) of this model still run the per-operator kernels: destroy them first", m->operator_contexts.load());
    return SSD_ESTATE;
  }
  SSD_HIP(hipDeviceSynchronize());   // nothing enqueued may still read them
  for (ssd_model::Layer& L : m->layers) {
    for (void** w : {&L.wqkv, &L.wo, &L.w_gate, &L.w_up, &L.w_down}) {
      if (*w) m->arena.release_one(*w);
      *w = nullptr;
    }
  }
  if (m->lm_head && m->lm_head != m->embed) m->arena.release_one(m->lm_head);
  m->lm_head = nullptr;
  m->operator_weights = false;
  return SSD_OK;
}

int ssd_model_destroy(ssd_model* m) {
  if (!m) return SSD_OK;
  m->arena.release();
  delete m;
  return SSD_OK;
}

}  // extern "C"

// One context for both cache shapes: h_fanout == nullptr is the uniform F of the configuration.
static int ctx_create(const ssd_model* model, const ssd_round_config* cfg, const int32_t* h_fanout, ssd_ctx** out) {
  SSD_CHECK_ARG(model && cfg && out, "ssd_ctx_create: null argument");
  *out = nullptr;
  SSD_CHECK_ARG(cfg->batch >= 1, "batch must be >= 1");
  SSD_CHECK_ARG(cfg->K >= 1 && cfg->K <= SSD_MAX_K, "K must be in 1..%d", SSD_MAX_K);
  SSD_CHECK_ARG(cfg->max_trunk >= 2 * cfg->K + 3, "max_trunk must be at least 2K+3");
  SSD_CHECK_ARG((cfg->flags & ~(SSD_CTX_PER_OPERATOR | SSD_CTX_FUSED_PHASES | SSD_CTX_NARROW_PASSES | SSD_CTX_ONE_PLANE_ALL | SSD_CTX_TWO_PLANES)) == 0,
                "unknown bits in ssd_round_config.flags");
  FanTable fan = {};
  int f_max = 0;
  for (int k = 0; k <= cfg->K; ++k) {
    const int f = h_fanout ? h_fanout[k] : cfg->F;
    SSD_CHECK_ARG(f >= 1 && f <= SSD_MAX_F, "fan-out %d at accept length %d: must be in 1..%d", f, k, SSD_MAX_F);
    fan.off[k + 1] = fan.off[k] + f;
    f_max = f > f_max ? f : f_max;
  }
  SSD_CHECK_ARG(f_max + 1 <= model->dims.vocab, "F + 1 must not exceed the vocabulary");
  SSD_CHECK_ARG((int64_t)cfg->batch * fan.off[cfg->K + 1] <= (1 << 20), "too many branch rows");
  ssd_ctx* c = new (std::nothrow) ssd_ctx();
  if (!c) { set_error("out of host memory"); return SSD_ENOMEM; }
  const Dims& d = model->dims;
  c->model = model; c->B = cfg->batch; c->K = cfg->K; c->F = f_max; c->max_trunk = cfg->max_trunk;
  c->fan = fan; c->rows_per_seq = fan.off[c->K + 1];
  c->M = c->B * c->rows_per_seq;
  c->max_rows = c->M > c->B * (c->K + 1) ? c->M : c->B * (c->K + 1);
  const size_t es = elem_size(d.dtype);
  const size_t kvd = (size_t)d.kv_dim();
  const int R = c->max_rows;
  int st = SSD_OK;
  auto A = [&](void** p, size_t bytes) { if (st == SSD_OK) st = c->arena.alloc(p, bytes); };
  A((void**)&c->trunk_len, sizeof(int32_t) * c->B);
  c->trunk_k.resize(d.n_layers); c->trunk_v.resize(d.n_layers);
  c->suffix_k.resize(d.n_layers); c->suffix_v.resize(d.n_layers);
  // the fused pass serves every pass of a context it fits, unless the configuration's flags say otherwise
  c->flags = cfg->flags;
  // (narrow passes of at most kFusedMaxRows rows in one persistent launch; a context with more rows in a batched
  // forward takes wide passes, one launch per phase, if the model's shape allows, else narrow passes of whole sequences,
  // else one kernel per operator)
  {
    const bool attn_ok = (16 / (d.n_q_heads / d.n_kv_heads)) * (c->K + 1 <= 8 ? 8 : 16) <= 64;
    const bool narrow_ok = model->fused_ok && fused_supported(d, c->rows_per_seq) && attn_ok;
    const bool wide_ok = model->wide_ok && attn_ok && c->max_rows > kFusedMaxRows && c->rows_per_seq <= kFusedWideRows &&
                         c->K + 1 <= kFusedWideRows;
    c->fused_mode = 0;
    c->fused_cap = kFusedMaxRows;
    if (cfg->flags & SSD_CTX_PER_OPERATOR) {
    } else if (wide_ok && !(cfg->flags & SSD_CTX_NARROW_PASSES)) {
      c->fused_mode = 1;
      c->fused_wide = true;
      c->fused_cap = kFusedWideRows;
    } else if (narrow_ok) {
      c->fused_mode = (cfg->flags & SSD_CTX_FUSED_PHASES) ? 1 : 2;
    }
  }
  if (!c->fused_mode) {
    if (!model->operator_weights) {
      set_error("this context would run the per-operator kernels (flags, or a shape the fused passes do not take), whose "
                "weights were released (ssd_model_release_operator_weights)");
      c->arena.release();
      delete c;
      return SSD_ESTATE;
    }
    model->operator_contexts.fetch_add(1);
  }
  c->vt_stride = (c->max_trunk + 63) / 64 * 64;
  c->ub_of.assign(c->B, 0);
  c->blocks_of.assign(c->B, 0);
  if (cfg->kv_pages) {
    // paged trunk (App. B): a pool of 32-position pages per layer instead of max_trunk positions per sequence
    if (!c->fused_mode || d.head_dim != 64) {
      set_error("kv_pages: the paged trunk is served by the fused passes only (bf16 model of a supported shape, no SSD_CTX_PER_OPERATOR)");
      ssd_ctx_destroy(c);
      return SSD_EINVAL;
    }
    if (cfg->kv_pages < 2 || c->max_trunk > 16384) {
      set_error("kv_pages must be at least 2 (page 0 is the shared all-zero page) and max_trunk at most 16384 in a paged context");
      ssd_ctx_destroy(c);
      return SSD_EINVAL;
    }
    c->kv_pages = cfg->kv_pages;
    c->page_stride = c->vt_stride / 32;
    // pages are handed out from the back of the list: low ids first
    for (int pg = c->kv_pages - 1; pg >= 1; --pg) c->free_pages.push_back(pg);
    A((void**)&c->page_table_dev, sizeof(int32_t) * (size_t)c->B * c->page_stride);
    if (st == SSD_OK) {
      void* host = nullptr;
      hipError_t e = hipHostMalloc(&host, sizeof(int32_t) * (size_t)c->B * c->page_stride, hipHostMallocDefault);
      if (e != hipSuccess) { (void)hipGetLastError(); set_error("hipHostMalloc failed: %s", hipGetErrorString(e)); st = SSD_ENOMEM; }
      else {
        c->page_table_host = (int32_t*)host;
        memset(host, 0, sizeof(int32_t) * (size_t)c->B * c->page_stride);
        hipError_t e2 = hipMemset(c->page_table_dev, 0, sizeof(int32_t) * (size_t)c->B * c->page_stride);
        if (e2 != hipSuccess) { set_error("hipMemset failed: %s", hipGetErrorString(e2)); st = SSD_EHIP; }
      }
    }
  }
  for (int l = 0; l < d.n_layers; ++l) {
    // fused contexts keep the trunk head-major, with max_trunk rounded up to 64 positions (layouts in fused.h)
    const size_t trunk_pos = c->fused_mode ? (size_t)c->vt_stride : (size_t)c->max_trunk;
    const size_t trunk_elems = c->kv_pages ? (size_t)c->kv_pages * 32 * kvd : (size_t)c->B * trunk_pos * kvd;
    A(&c->trunk_k[l], trunk_elems * es);
    A(&c->trunk_v[l], trunk_elems * es);
    A(&c->suffix_k[l], (size_t)c->M * c->K * kvd * es);
    A(&c->suffix_v[l], (size_t)c->M * c->K * kvd * es);
  }
  A((void**)&c->keys, sizeof(int32_t) * c->M);
  A((void**)&c->tokens, sizeof(int32_t) * c->M * c->K);
  A((void**)&c->logits, sizeof(float) * (size_t)c->M * c->K * d.vocab);
  A((void**)&c->hidden, sizeof(float) * (size_t)c->M * c->K * d.d_model);
  A((void**)&c->glue_logits, sizeof(float) * (size_t)c->B * (c->K + 1) * d.vocab);
  A((void**)&c->glue_hidden, sizeof(float) * (size_t)c->B * (c->K + 1) * d.d_model);
  A((void**)&c->rows, sizeof(RowDesc) * R);
  A((void**)&c->cos_sin, sizeof(float) * (size_t)R * d.head_dim);
  A((void**)&c->step_tokens, sizeof(int32_t) * R);
  A((void**)&c->exclude, sizeof(int32_t) * c->B * (c->K + 1));
  A((void**)&c->h, sizeof(float) * (size_t)R * d.d_model);
  A(&c->xn, sizeof(float) * (size_t)R * d.d_model);
  A((void**)&c->qkv, sizeof(float) * (size_t)R * d.qkv_dim());
  A((void**)&c->q, sizeof(float) * (size_t)R * d.q_dim());
  A(&c->attn_out, sizeof(float) * (size_t)R * d.q_dim());
  A(&c->act, sizeof(float) * (size_t)R * d.d_ffn);
  c->attn_partial_floats = attention_partial_floats(R, d.n_q_heads, d.head_dim, c->max_trunk + c->K);
  A((void**)&c->attn_partial, (size_t)c->attn_partial_floats * sizeof(float));
  A(&c->sample_scratch, sample_scratch_bytes(c->M));
  A(&c->top_f_scratch, top_f_scratch_bytes(R));
  A((void**)&c->sigma_ids, sizeof(int32_t) * (size_t)c->M * c->F);
  if (st == SSD_OK && c->fused_mode) st = fused_setup(c);
  if (st == SSD_OK) {
    hipError_t e = hipMemset(c->trunk_len, 0, sizeof(int32_t) * c->B);
    if (e != hipSuccess) { set_error("hipMemset failed: %s", hipGetErrorString(e)); st = SSD_EHIP; }
  }
  if (st != SSD_OK) { ssd_ctx_destroy(c); return st; }
  *out = c;
  return SSD_OK;
}

extern "C" {

int ssd_ctx_create(const ssd_model* model, const ssd_round_config* cfg, ssd_ctx** out) {
  return ctx_create(model, cfg, nullptr, out);
}

int ssd_ctx_create_fanout(const ssd_model* model, const ssd_round_config* cfg, const int32_t* h_fanout, ssd_ctx** out) {
  SSD_CHECK_ARG(h_fanout, "ssd_ctx_create_fanout: null fan-out");
  return ctx_create(model, cfg, h_fanout, out);
}

int ssd_ctx_fanout(const ssd_ctx* c, int32_t* h_fanout) {
  SSD_CHECK_ARG(c && h_fanout, "ssd_ctx_fanout: null argument");
  for (int k = 0; k <= c->K; ++k) h_fanout[k] = c->fan.off[k + 1] - c->fan.off[k];
  return SSD_OK;
}

int ssd_geometric_fanout(int32_t budget, int32_t K, double a, double r, int32_t f_max, int32_t* h_fanout) {
  SSD_CHECK_ARG(h_fanout, "ssd_geometric_fanout: null output");
  SSD_CHECK_ARG(K >= 0 && K <= SSD_MAX_K, "K must be in 0..%d", SSD_MAX_K);
  SSD_CHECK_ARG(a > 0.0 && a < 1.0 && r > 0.0, "acceptance rate in (0,1) and power-law exponent > 0 required");
  SSD_CHECK_ARG(f_max >= 1 && budget >= K + 1 && (int64_t)budget <= (int64_t)(K + 1) * f_max,
                "budget %d must lie between K+1 and (K+1) f_max", budget);
  const int n = K + 1;
  // the theorem's proportions: a^(k/(1+r)), the last one larger by (1-a)^(-1/(1+r))
  double w[SSD_MAX_K + 1], x[SSD_MAX_K + 1];
  const double q = pow(a, 1.0 / (1.0 + r));
  for (int k = 0; k < n; ++k) w[k] = pow(q, (double)k);
  w[K] *= pow(1.0 - a, -1.0 / (1.0 + r));
  // bounds 1..f_max: an accept length the proportions put outside is held at the bound and the others share the rest
  int state[SSD_MAX_K + 1] = {};   // 0 free, 1 at the lower bound, 2 at the upper
  for (;;) {
    double left = budget, wsum = 0.0;
    for (int k = 0; k < n; ++k) {
      if (state[k] == 1) left -= 1.0;
      else if (state[k] == 2) left -= f_max;
      else wsum += w[k];
    }
    bool over = false, under = false;
    for (int k = 0; k < n; ++k) {
      x[k] = state[k] == 1 ? 1.0 : state[k] == 2 ? (double)f_max : left * w[k] / wsum;
      over |= state[k] == 0 && x[k] > f_max;
      under |= state[k] == 0 && x[k] < 1.0;
    }
    if (over) { for (int k = 0; k < n; ++k) if (state[k] == 0 && x[k] > f_max) state[k] = 2; }
    else if (under) { for (int k = 0; k < n; ++k) if (state[k] == 0 && x[k] < 1.0) state[k] = 1; }
    else break;
  }
  // largest remainders take the units the floors leave over (lower accept length first on ties)
  int total = 0;
  double frac[SSD_MAX_K + 1];
  for (int k = 0; k < n; ++k) {
    h_fanout[k] = (int32_t)floor(x[k] + 1e-9);
    frac[k] = x[k] - h_fanout[k];
    total += h_fanout[k];
  }
  for (int spare = budget - total; spare > 0; --spare) {
    int best = -1;
    for (int k = 0; k < n; ++k)
      if (h_fanout[k] < f_max && (best < 0 || frac[k] > frac[best])) best = k;
    h_fanout[best] += 1;
    frac[best] = -1.0;
  }
  return SSD_OK;
}

int ssd_ctx_destroy(ssd_ctx* c) {
  if (!c) return SSD_OK;
  {
    // a later persistent launch must not wait on an event that no longer exists
    std::lock_guard<std::mutex> lock(g_fused_mu);
    if (g_fused_last_ctx == c) {
      (void)hipEventSynchronize(c->fused_done);
      g_fused_last_event = nullptr;
      g_fused_last_stream = nullptr;
      g_fused_last_ctx = nullptr;
    }
  }
  if (!c->fused_mode && c->model) c->model->operator_contexts.fetch_sub(1);
  if (c->fused_done) (void)hipEventDestroy(c->fused_done);
  if (c->fused_err) (void)hipHostFree(c->fused_err);
  if (c->page_table_host) (void)hipHostFree(c->page_table_host);
  for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
  for (hipEvent_t e : c->kernel_events) (void)hipEventDestroy(e);
  c->arena.release();
  delete c;
  return SSD_OK;
}

int ssd_ctx_prefill(ssd_ctx* c, const int32_t* d_tokens, int32_t stride, const int32_t* h_lens, void* stream) {
  SSD_CHECK_ARG(c && d_tokens && h_lens, "ssd_ctx_prefill: null argument");
  SSD_TRY(ctx_fault(c, "ssd_ctx_prefill"));
  hipStream_t s = (hipStream_t)stream;
  int max_len = 0;
  for (int b = 0; b < c->B; ++b) {
    SSD_CHECK_ARG(h_lens[b] >= 1 && h_lens[b] <= stride, "prefill length %d of sequence %d out of range", h_lens[b], b);
    max_len = h_lens[b] > max_len ? h_lens[b] : max_len;
  }
  SSD_CHECK_ARG(max_len + 2 * c->K + 2 <= c->max_trunk, "prefill of %d tokens does not leave room for a round (max_trunk %d)",
                max_len, c->max_trunk);
  SSD_TRY(launch_fill_i32(c->trunk_len, 0, c->B, s));
  const int T = c->K + 1;
  {
    std::vector<int32_t> zero(c->B, 0);
    set_bounds(c, zero.data());
    if (c->kv_pages) {       // the new text starts from an empty trunk: every page goes back first
      SSD_HIP(hipStreamSynchronize(s));
      bool dirty = false;
      for (int b = 0; b < c->B; ++b) pages_release_beyond(c, b, 0, &dirty);
    }
  }
  for (int start = 0; start < max_len; start += T) {
    int n = c->B * T;
    gather_chunk_tokens_kernel<<<(n + 255) / 256, 256, 0, s>>>(c->step_tokens, d_tokens, stride, c->B, T, start);
    SSD_HIP(hipGetLastError());
    SSD_TRY(extend_rows(c, c->step_tokens, T, start, nullptr, nullptr, 0, c->B, s));
  }
  SSD_HIP(hipMemcpyAsync(c->trunk_len, h_lens, sizeof(int32_t) * c->B, hipMemcpyHostToDevice, s));
  SSD_HIP(hipStreamSynchronize(s));   // h_lens is caller-owned pageable memory
  set_bounds(c, h_lens);
  if (c->kv_pages) {         // the chunks ran to the longest prompt: shorter ones hand the surplus back
    bool dirty = false;
    for (int b = 0; b < c->B; ++b) pages_release_beyond(c, b, h_lens[b], &dirty);
    if (dirty) SSD_TRY(pages_upload(c, s));
  }
  c->have_cache = false;
  return SSD_OK;
}

int ssd_ctx_prefill_sequence(ssd_ctx* c, int32_t b, const int32_t* d_tokens, int32_t len, void* stream) {
  SSD_CHECK_ARG(c && d_tokens, "ssd_ctx_prefill_sequence: null argument");
  SSD_CHECK_ARG(b >= 0 && b < c->B, "ssd_ctx_prefill_sequence: sequence %d out of range", b);
  SSD_CHECK_ARG(len >= 1 && len + 2 * c->K + 2 <= c->max_trunk, "prefill of %d tokens does not leave room for a round (max_trunk %d)",
                len, c->max_trunk);
  SSD_TRY(ctx_fault(c, "ssd_ctx_prefill_sequence"));
  hipStream_t s = (hipStream_t)stream;
  SSD_HIP(hipStreamSynchronize(s));
  {
    bool dirty = false;
    pages_release_beyond(c, b, 0, &dirty);
    if (dirty) SSD_TRY(pages_upload(c, s));
  }
  SSD_TRY(launch_fill_i32(c->trunk_len + b, 0, 1, s));
  c->ub_of[b] = 0;
  const int T = c->K + 1;
  for (int start = 0; start < len; start += T) {
    gather_chunk_tokens_kernel<<<1, 256, 0, s>>>(c->step_tokens, d_tokens, len, 1, T, start);
    SSD_HIP(hipGetLastError());
    SSD_TRY(extend_rows(c, c->step_tokens, T, start, nullptr, nullptr, b, 1, s));
  }
  SSD_TRY(launch_fill_i32(c->trunk_len + b, len, 1, s));
  c->ub_of[b] = len;
  if (c->kv_pages) {
    SSD_HIP(hipStreamSynchronize(s));
    bool dirty = false;
    pages_release_beyond(c, b, len, &dirty);
    if (dirty) SSD_TRY(pages_upload(c, s));
  }
  c->trunk_ub = 0;
  for (int i = 0; i < c->B; ++i) c->trunk_ub = c->ub_of[i] > c->trunk_ub ? c->ub_of[i] : c->trunk_ub;
  c->have_cache = false;
  return SSD_OK;
}

int ssd_ctx_release_sequence(ssd_ctx* c, int32_t b, void* stream) {
  SSD_CHECK_ARG(c, "ssd_ctx_release_sequence: null context");
  SSD_CHECK_ARG(b >= 0 && b < c->B, "ssd_ctx_release_sequence: sequence %d out of range", b);
  hipStream_t s = (hipStream_t)stream;
  SSD_HIP(hipStreamSynchronize(s));
  bool dirty = false;
  pages_release_beyond(c, b, 0, &dirty);
  if (dirty) SSD_TRY(pages_upload(c, s));
  SSD_TRY(launch_fill_i32(c->trunk_len + b, 0, 1, s));
  c->ub_of[b] = 0;
  c->trunk_ub = 0;
  for (int i = 0; i < c->B; ++i) c->trunk_ub = c->ub_of[i] > c->trunk_ub ? c->ub_of[i] : c->trunk_ub;
  c->have_cache = false;
  return SSD_OK;
}

int ssd_ctx_kv_pages(const ssd_ctx* c, int32_t* total, int32_t* free_pages) {
  SSD_CHECK_ARG(c && total && free_pages, "ssd_ctx_kv_pages: null argument");
  *total = c->kv_pages;
  *free_pages = (int32_t)c->free_pages.size();
  return SSD_OK;
}

int ssd_ctx_load_trunk(ssd_ctx* c, const void* d_k, const void* d_v, int32_t len, void* stream) {
  SSD_CHECK_ARG(c && d_k && d_v, "ssd_ctx_load_trunk: null argument");
  SSD_CHECK_ARG(len >= 1 && len + 2 * c->K + 2 <= c->max_trunk, "trunk length %d does not fit max_trunk %d with room for a round",
                len, c->max_trunk);
  hipStream_t s = (hipStream_t)stream;
  const Dims& d = c->model->dims;
  const size_t es = elem_size(d.dtype);
  const size_t per_layer = (size_t)c->B * len * d.kv_dim() * es;
  if (c->kv_pages) {
    bool dirty = false;
    for (int b = 0; b < c->B; ++b) SSD_TRY(pages_ensure(c, b, len, &dirty));
    if (dirty) SSD_TRY(pages_upload(c, s));
  }
  for (int l = 0; l < d.n_layers; ++l) {
    if (c->fused_mode) {
      SSD_TRY(launch_copy_kv_fused((bf16_t*)c->trunk_k[l], (bf16_t*)c->trunk_v[l], (const bf16_t*)((const char*)d_k + l * per_layer),
                                   (const bf16_t*)((const char*)d_v + l * per_layer), c->B, len, d.n_kv_heads, c->vt_stride,
                                   c->kv_pages ? c->page_table_dev : nullptr, c->page_stride, s));
    } else {
      SSD_TRY(launch_copy_kv_in(d.dtype, c->trunk_k[l], (const char*)d_k + l * per_layer, c->B, len, c->max_trunk, d.kv_dim(), s));
      SSD_TRY(launch_copy_kv_in(d.dtype, c->trunk_v[l], (const char*)d_v + l * per_layer, c->B, len, c->max_trunk, d.kv_dim(), s));
    }
  }
  SSD_TRY(launch_fill_i32(c->trunk_len, len, c->B, s));
  {
    std::vector<int32_t> lens(c->B, len);
    set_bounds(c, lens.data());
  }
  c->have_cache = false;
  return SSD_OK;
}

int ssd_ctx_fill_synthetic_kv(ssd_ctx* c, const int32_t* h_lens, uint64_t seed, void* stream) {
  SSD_CHECK_ARG(c && h_lens, "ssd_ctx_fill_synthetic_kv: null argument");
  SSD_TRY(ctx_fault(c, "ssd_ctx_fill_synthetic_kv"));
  int max_len = 0;
  for (int b = 0; b < c->B; ++b) {
    SSD_CHECK_ARG(h_lens[b] >= 1 && h_lens[b] + 2 * c->K + 2 <= c->max_trunk,
                  "synthetic prefix of %d positions for sequence %d does not fit max_trunk %d with room for a round", h_lens[b], b,
                  c->max_trunk);
    max_len = h_lens[b] > max_len ? h_lens[b] : max_len;
  }
  hipStream_t s = (hipStream_t)stream;
  const Dims& d = c->model->dims;
  SSD_HIP(hipMemcpyAsync(c->trunk_len, h_lens, sizeof(int32_t) * c->B, hipMemcpyHostToDevice, s));
  SSD_HIP(hipStreamSynchronize(s));   // h_lens is caller-owned pageable memory
  if (c->kv_pages) {
    bool dirty = false;
    for (int b = 0; b < c->B; ++b) {
      pages_release_beyond(c, b, h_lens[b], &dirty);
      SSD_TRY(pages_ensure(c, b, h_lens[b], &dirty));
    }
    if (dirty) SSD_TRY(pages_upload(c, s));
  }
  for (int l = 0; l < d.n_layers; ++l)
    SSD_TRY(launch_fill_kv(d.dtype, c->trunk_k[l], c->trunk_v[l], c->trunk_len, c->B, max_len, d.n_kv_heads, d.head_dim,
                           c->fused_mode ? c->vt_stride : c->max_trunk, c->fused_mode ? 1 : 0,
                           c->kv_pages ? c->page_table_dev : nullptr, c->page_stride, seed, (1ull << 20) + 2 * (uint64_t)l,
                           (1ull << 20) + 2 * (uint64_t)l + 1, s));
  set_bounds(c, h_lens);
  c->have_cache = false;
  return SSD_OK;
}

int ssd_ctx_truncate_trunk(ssd_ctx* c, const int32_t* h_lens, void* stream) {
  SSD_CHECK_ARG(c && h_lens, "ssd_ctx_truncate_trunk: null argument");
  for (int b = 0; b < c->B; ++b)
    SSD_CHECK_ARG(h_lens[b] >= 1 && h_lens[b] <= c->trunk_ub && (!c->kv_pages || h_lens[b] <= c->ub_of[b]),
                  "trunk length %d of sequence %d: must be in 1..%d", h_lens[b], b, c->kv_pages ? c->ub_of[b] : c->trunk_ub);
  hipStream_t s = (hipStream_t)stream;
  SSD_HIP(hipMemcpyAsync(c->trunk_len, h_lens, sizeof(int32_t) * c->B, hipMemcpyHostToDevice, s));
  SSD_HIP(hipStreamSynchronize(s));   // h_lens is caller-owned pageable memory
  set_bounds(c, h_lens);
  if (c->kv_pages) {
    bool dirty = false;
    for (int b = 0; b < c->B; ++b) pages_release_beyond(c, b, h_lens[b], &dirty);
    if (dirty) SSD_TRY(pages_upload(c, s));
  }
  c->have_cache = false;
  return SSD_OK;
}

int ssd_ctx_set_forced(ssd_ctx* c, const int32_t* d_keys, const int32_t* d_tokens) {
  SSD_CHECK_ARG(c, "ssd_ctx_set_forced: null context");
  c->forced_keys = d_keys;
  c->forced_tokens = d_tokens;
  return SSD_OK;
}

int ssd_ctx_extend(ssd_ctx* c, const int32_t* d_tokens, int32_t T, int32_t offset, float* d_logits, void* stream) {
  SSD_CHECK_ARG(c && d_tokens, "ssd_ctx_extend: null argument");
  SSD_CHECK_ARG(T >= 1 && T <= c->K + 1, "extend of %d tokens: must be in 1..K+1", T);
  SSD_CHECK_ARG(offset >= 0, "negative offset");
  SSD_TRY(ctx_fault(c, "ssd_ctx_extend"));
  if (c->trunk_ub + offset + T > c->max_trunk) {
    set_error("extend would pass max_trunk (%d + %d + %d > %d)", c->trunk_ub, offset, T, c->max_trunk);
    return SSD_ESTATE;
  }
  return extend_rows(c, d_tokens, T, offset, d_logits, nullptr, 0, c->B, (hipStream_t)stream);
}

int ssd_prespeculate(ssd_ctx* c, const int32_t* d_pending, const float* d_temperature, uint64_t round_seed, void* stream) {
  SSD_CHECK_ARG(c && d_pending && d_temperature, "ssd_prespeculate: null argument");
  SSD_TRY(ctx_fault(c, "ssd_prespeculate"));
  if (c->trunk_ub < 1) { set_error("ssd_prespeculate: the trunk is empty (prefill or load it first)"); return SSD_ESTATE; }
  for (int b = 0; b < c->B; ++b)
    if (c->ub_of[b] < 1) { set_error("ssd_prespeculate: the trunk of sequence %d is empty (prefill its slot first)", b); return SSD_ESTATE; }
  if (c->trunk_ub + 2 * c->K + 2 > c->max_trunk) {
    set_error("ssd_prespeculate: trunk bound %d + 2K+2 exceeds max_trunk %d", c->trunk_ub, c->max_trunk);
    return SSD_ESTATE;
  }
  hipStream_t s = (hipStream_t)stream;
  const Dims& d = c->model->dims;
  const int K = c->K, B = c->B, M = c->M, V = d.vocab, RB = c->rows_per_seq;
  int ev = 0;
  auto mark = [&]() -> int {
    if (c->timing) SSD_HIP(hipEventRecord(c->events[ev++], s));
    return SSD_OK;
  };
  SSD_TRY(mark());
  // a0: glue extend of {last verified token, s_1..s_K}
  SSD_TRY(extend_rows(c, d_pending, K + 1, 0, c->glue_logits, c->glue_hidden, 0, B, s));
  SSD_TRY(mark());
  // a1: fan-out
  SSD_TRY(launch_pending_exclude(c->exclude, d_pending, B, K, s));
  SSD_TRY(launch_top_f_fan(c->glue_logits, V, c->exclude, B, K, c->fan, V, c->keys, c->top_f_scratch, s));
  SSD_TRY(mark());
  // a2/a3: K batched branch-decode steps; logits and tokens land in the cache directly
  for (int i = 0; i < K; ++i) {
    SSD_TRY(launch_setup_branch_rows(c->rows, c->cos_sin, c->trunk_len, B, K, c->fan, i, d.head_dim / 2, d.rope_theta, c->step_tokens,
                                     c->keys, c->tokens, c->forced_keys, c->forced_tokens, s));
    SSD_TRY(forward_rows(c, M, c->step_tokens, RB, c->trunk_ub + K + 1, i, c->logits + (size_t)i * V, (int64_t)K * V,
                         c->hidden + (size_t)i * d.d_model, (int64_t)K * d.d_model, 0, s));
    if (c->saguaro_c < 1.0f) {
      // sigma_{F,C}: lower the step's own top-F logits before the draw; the cache keeps the lowered logits, the
      // distribution the tokens are drawn from.  The token of depth i is the one whose rejection ends the next round
      // at accept length i, where the cache holds F_i candidates.
      const int F = c->fan.off[i + 1] - c->fan.off[i];
      SSD_TRY(launch_top_f(c->logits + (size_t)i * V, (int64_t)K * V, nullptr, M, V, F, c->sigma_ids, c->top_f_scratch, s));
      SSD_TRY(launch_sigma_shift(c->logits + (size_t)i * V, (int64_t)K * V, d_temperature, RB, M, F, c->sigma_ids,
                                 c->saguaro_c > 0.f ? logf(c->saguaro_c) : -INFINITY, s));
    }
    SSD_TRY(launch_sample(c->logits + (size_t)i * V, (int64_t)K * V, d_temperature, RB, M, V, round_seed, 0, i,
                          c->tokens + i, K, c->sample_scratch, 0, s));
    SSD_TRY(mark());
  }
  c->have_cache = true;
  return SSD_OK;
}

int ssd_cache_lookup(ssd_ctx* c, const int32_t* d_accept_len, const int32_t* d_bonus, uint8_t* d_hit, int32_t* d_branch,
                     int32_t* d_spec_tokens, const float** d_logits_ptr, void* stream) {
  SSD_CHECK_ARG(c && d_accept_len && d_bonus && d_hit && d_branch && d_spec_tokens, "ssd_cache_lookup: null argument");
  SSD_TRY(ctx_fault(c, "ssd_cache_lookup"));
  if (!c->have_cache) { set_error("ssd_cache_lookup before any ssd_prespeculate"); return SSD_ESTATE; }
  return launch_lookup(c->keys, c->tokens, c->logits, d_accept_len, d_bonus, d_hit, d_branch, d_spec_tokens, d_logits_ptr,
                       c->B, c->K, c->fan, c->model->dims.vocab, (hipStream_t)stream);
}

int ssd_ctx_commit(ssd_ctx* c, const int32_t* d_accept_len, void* stream) {
  SSD_CHECK_ARG(c && d_accept_len, "ssd_ctx_commit: null argument");
  SSD_TRY(ctx_fault(c, "ssd_ctx_commit"));
  if (c->trunk_ub < 1) { set_error("ssd_ctx_commit: the trunk is empty"); return SSD_ESTATE; }
  SSD_TRY(launch_commit(c->trunk_len, d_accept_len, c->B, c->K, (hipStream_t)stream));
  c->trunk_ub += c->K + 1;
  for (int b = 0; b < c->B; ++b) c->ub_of[b] += c->K + 1;
  return SSD_OK;
}

int ssd_ctx_set_saguaro(ssd_ctx* c, float C) {
  SSD_CHECK_ARG(c, "ssd_ctx_set_saguaro: null context");
  SSD_CHECK_ARG(C >= 0.f && C <= 1.f, "the downweighting constant must be in [0, 1]");
  c->saguaro_c = C;
  return SSD_OK;
}

int ssd_ctx_refresh_bounds(ssd_ctx* c, void* stream) {
  SSD_CHECK_ARG(c, "ssd_ctx_refresh_bounds: null context");
  std::vector<int32_t> lens(c->B);
  SSD_HIP(hipMemcpyAsync(lens.data(), c->trunk_len, sizeof(int32_t) * c->B, hipMemcpyDeviceToHost, (hipStream_t)stream));
  SSD_HIP(hipStreamSynchronize((hipStream_t)stream));
  set_bounds(c, lens.data());
  if (c->kv_pages) {
    // page rollback: the pages behind a sequence's verified text (rejected tokens' positions, old glue) return to the pool
    bool dirty = false;
    for (int b = 0; b < c->B; ++b) pages_release_beyond(c, b, lens[b], &dirty);
    if (dirty) SSD_TRY(pages_upload(c, (hipStream_t)stream));
  }
  return ctx_fault(c, "ssd_ctx_refresh_bounds");
}

int ssd_ctx_status(const ssd_ctx* c) {
  SSD_CHECK_ARG(c, "ssd_ctx_status: null context");
  return ctx_fault(c, "ssd_ctx_status");
}

int ssd_ctx_recover(ssd_ctx* c) {
  SSD_CHECK_ARG(c, "ssd_ctx_recover: null context");
  SSD_HIP(hipDeviceSynchronize());
  if (c->fused_mode) {
    SSD_TRY(fused_init_barrier(c->fused_bar, 0u, c->fp.nwg));
    SSD_TRY(fused_init_group_flags(c->fp.qkv_flags, c->fp.L, 0u));
    SSD_HIP(hipMemset(c->fp.fix_buf, 0xff, (size_t)c->fp.L * 3 * c->fp.fix_stride * 4));
    SSD_HIP(hipMemset(c->fp.arrivals, 0, (size_t)c->fp.L * c->fp.arrivals_stride * 4));
    *(volatile unsigned*)c->fused_err = 0u;
  }
  c->have_cache = false;
  return SSD_OK;
}

int ssd_ctx_debug_set(ssd_ctx* c, int32_t what, uint32_t value) {
  SSD_CHECK_ARG(c, "ssd_ctx_debug_set: null context");
  if (!c->fused_mode) { set_error("ssd_ctx_debug_set: the context is not served by the fused pass"); return SSD_ESTATE; }
  if (what == SSD_DEBUG_BARRIER_EPOCH) {
    SSD_HIP(hipDeviceSynchronize());
    SSD_TRY(fused_init_group_flags(c->fp.qkv_flags, c->fp.L, value));
    return fused_init_barrier(c->fused_bar, value, c->fp.nwg);
  }
  if (what == SSD_DEBUG_SPIN_LIMIT) {
    c->fp.spin_limit = value ? value : kFusedSpinLimit;
    return SSD_OK;
  }
  set_error("ssd_ctx_debug_set: unknown item %d", what);
  return SSD_EINVAL;
}

int ssd_ctx_enable_timing(ssd_ctx* c, int32_t on) {
  SSD_CHECK_ARG(c, "ssd_ctx_enable_timing: null context");
  if (on && c->events.empty()) {
    for (int i = 0; i < c->K + 3; ++i) {
      hipEvent_t e;
      SSD_HIP(hipEventCreate(&e));
      c->events.push_back(e);
    }
    for (int i = 0; c->fused_mode && i < 2 * c->K; ++i) {
      hipEvent_t e;
      SSD_HIP(hipEventCreate(&e));
      c->kernel_events.push_back(e);
    }
  }
  c->timing = on != 0;
  return SSD_OK;
}

int ssd_ctx_enable_phase_clocks(ssd_ctx* c, int32_t on) {
  SSD_CHECK_ARG(c, "ssd_ctx_enable_phase_clocks: null context");
  if (!c->fused_mode) { set_error("phase clocks exist only in contexts served by the fused pass"); return SSD_ESTATE; }
  if (on && !c->phase_clocks) {
    const size_t n = (size_t)(fused_last_phase(c->fp.L) + 1) * kFusedClockSlots * c->fp.nwg;
    SSD_TRY(c->arena.alloc((void**)&c->phase_clocks, n * sizeof(unsigned long long)));
    SSD_HIP(hipMemset(c->phase_clocks, 0, n * sizeof(unsigned long long)));
  }
  c->fp.prof = on ? c->phase_clocks : nullptr;
  return SSD_OK;
}

int ssd_ctx_read_phase_clocks(ssd_ctx* c, uint64_t* h_ticks, int64_t n, int32_t* n_phases, int32_t* n_workgroups) {
  SSD_CHECK_ARG(c && h_ticks && n_phases && n_workgroups, "ssd_ctx_read_phase_clocks: null argument");
  if (!c->phase_clocks) { set_error("phase clocks are not enabled"); return SSD_ESTATE; }
  *n_phases = fused_last_phase(c->fp.L) + 1;
  *n_workgroups = c->fp.nwg;
  const int64_t need = (int64_t)*n_phases * kFusedClockSlots * c->fp.nwg;
  SSD_CHECK_ARG(n >= need, "ssd_ctx_read_phase_clocks: buffer of %lld entries, %lld needed", (long long)n, (long long)need);
  SSD_HIP(hipDeviceSynchronize());
  SSD_HIP(hipMemcpy(h_ticks, c->phase_clocks, (size_t)need * sizeof(uint64_t), hipMemcpyDeviceToHost));
  return SSD_OK;
}

int ssd_ctx_read_timing(ssd_ctx* c, float* h_ms, int32_t n) {
  SSD_CHECK_ARG(c && h_ms, "ssd_ctx_read_timing: null argument");
  const bool with_kernels = n == 2 * c->K + 2 && !c->kernel_events.empty();
  SSD_CHECK_ARG(n == c->K + 2 || with_kernels, "ssd_ctx_read_timing: n must be K+2 (or 2K+2 in a context served by the fused pass)");
  if (!c->timing || !c->have_cache) { set_error("ssd_ctx_read_timing: no timed round has run"); return SSD_ESTATE; }
  SSD_HIP(hipEventSynchronize(c->events[c->K + 2]));
  SSD_TRY(ctx_fault(c, "ssd_ctx_read_timing"));
  for (int i = 0; i < c->K + 2; ++i) SSD_HIP(hipEventElapsedTime(&h_ms[i], c->events[i], c->events[i + 1]));
  for (int i = 0; with_kernels && i < c->K; ++i)
    SSD_HIP(hipEventElapsedTime(&h_ms[c->K + 2 + i], c->kernel_events[2 * i], c->kernel_events[2 * i + 1]));
  return SSD_OK;
}

size_t ssd_verify_workspace_bytes(int32_t B, int32_t K) {
  if (B < 1 || K < 1) return 0;
  return verify_workspace_bytes(B, K);
}

int ssd_verify(const float* d_target_logits, const float* d_draft_logits, const int32_t* d_spec_tokens,
               const float* d_temperature, int32_t B, int32_t K, int32_t V, uint64_t seed, int32_t* d_accept_len,
               int32_t* d_bonus, void* d_workspace, void* stream) {
  SSD_CHECK_ARG(d_target_logits && d_spec_tokens && d_temperature && d_accept_len && d_bonus && d_workspace,
                "ssd_verify: null argument");
  SSD_CHECK_ARG(B >= 1 && K >= 1 && K <= SSD_MAX_K && V >= 2, "ssd_verify: B >= 1, 1 <= K <= %d, V >= 2 required", SSD_MAX_K);
  return launch_verify(d_target_logits, d_draft_logits, d_spec_tokens, d_temperature, B, K, V, seed, d_accept_len, d_bonus,
                       d_workspace, (hipStream_t)stream);
}

int ssd_verify_static(const float* d_target_logits, const float* d_draft_logits, const int32_t* d_spec_tokens,
                      const float* d_temperature, int32_t B, int32_t K, int32_t V, uint64_t seed, int32_t* d_accept_len,
                      int32_t* d_bonus, void* stream) {
  SSD_CHECK_ARG(d_target_logits && d_spec_tokens && d_temperature && d_accept_len && d_bonus, "ssd_verify_static: null argument");
  SSD_CHECK_ARG(B >= 1 && K >= 1 && K <= SSD_MAX_K && V >= 2, "ssd_verify_static: B >= 1, 1 <= K <= %d, V >= 2 required", SSD_MAX_K);
  return launch_verify_static(d_target_logits, d_draft_logits, d_spec_tokens, d_temperature, B, K, V, seed, d_accept_len,
                              d_bonus, (hipStream_t)stream);
}

size_t ssd_verify_static_capacity(void) { return verify_static_capacity(); }

size_t ssd_top_f_workspace_bytes(int32_t rows) { return rows > 0 ? top_f_scratch_bytes(rows) : 0; }

int ssd_top_f(const float* d_logits, int64_t ld, const int32_t* d_exclude, int32_t rows, int32_t V, int32_t F,
              int32_t* d_ids, void* d_workspace, void* stream) {
  SSD_CHECK_ARG(d_logits && d_ids, "ssd_top_f: null argument");
  SSD_CHECK_ARG(rows >= 0 && V >= 2 && ld >= V, "ssd_top_f: rows >= 0, V >= 2, ld >= V required");
  SSD_CHECK_ARG(F >= 1 && F <= SSD_MAX_F && F + 1 <= V, "ssd_top_f: F must be in 1..%d and F + 1 <= V", SSD_MAX_F);
  return launch_top_f(d_logits, ld, d_exclude, rows, V, F, d_ids, d_workspace, (hipStream_t)stream);
}

int ssd_sample(const float* d_logits, int64_t ld, const float* d_temperature, int32_t rows, int32_t V, uint64_t seed,
               int32_t row_base, int32_t step, int32_t* d_out, void* stream) {
  SSD_CHECK_ARG(d_logits && d_temperature && d_out, "ssd_sample: null argument");
  SSD_CHECK_ARG(rows >= 0 && V >= 2 && ld >= V, "ssd_sample: rows >= 0, V >= 2, ld >= V required");
  return launch_sample(d_logits, ld, d_temperature, 1, rows, V, seed, row_base, step, d_out, 1, nullptr, 0, (hipStream_t)stream);
}

int ssd_sample_fp64_scan(const float* d_logits, int64_t ld, const float* d_temperature, int32_t rows, int32_t V, uint64_t seed,
                         int32_t row_base, int32_t step, int32_t* d_out, void* stream) {
  SSD_CHECK_ARG(d_logits && d_temperature && d_out, "ssd_sample_fp64_scan: null argument");
  SSD_CHECK_ARG(rows >= 0 && V >= 2 && ld >= V, "ssd_sample_fp64_scan: rows >= 0, V >= 2, ld >= V required");
  return launch_sample(d_logits, ld, d_temperature, 1, rows, V, seed, row_base, step, d_out, 1, nullptr, 1, (hipStream_t)stream);
}

int ssd_backup_random(uint64_t seed, int32_t B, int32_t K, int32_t V, int32_t* d_tokens, void* stream) {
  SSD_CHECK_ARG(d_tokens, "ssd_backup_random: null argument");
  SSD_CHECK_ARG(B >= 0 && K >= 0 && V >= 1 && (int64_t)B * K <= (1 << 24), "ssd_backup_random: B, K >= 0, V >= 1 required");
  return launch_backup_random(d_tokens, B, K, V, seed, (hipStream_t)stream);
}

int ssd_ctx_views(const ssd_ctx* c, ssd_views* out) {
  SSD_CHECK_ARG(c && out, "ssd_ctx_views: null argument");
  out->d_trunk_len = c->trunk_len; out->d_keys = c->keys; out->d_tokens = c->tokens; out->d_logits = c->logits;
  out->d_hidden = c->hidden; out->d_glue_logits = c->glue_logits; out->d_glue_hidden = c->glue_hidden;
  out->h_trunk_k = (const void* const*)c->trunk_k.data(); out->h_trunk_v = (const void* const*)c->trunk_v.data();
  out->batch = c->B; out->K = c->K; out->F = c->F; out->vocab = c->model->dims.vocab; out->d_model = c->model->dims.d_model;
  out->max_trunk = c->max_trunk;
  out->fused_pass = c->fused_mode;
  out->pass_rows = c->fused_mode ? c->fused_cap : 0;
  return SSD_OK;
}

}  // extern "C"
