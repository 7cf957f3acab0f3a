// Shared declarations of the HIP library: error plumbing, element types, row descriptors and
// the launchers each kernel file exports to the round driver.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ssd.h"

namespace ssd {

void set_error(const char* fmt, ...);

#define SSD_HIP(expr)                                                                 \
  do {                                                                                \
    hipError_t e_ = (expr);                                                           \
    if (e_ != hipSuccess) {                                                           \
      ::ssd::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return SSD_EHIP;                                                                \
    }                                                                                 \
  } while (0)

#define SSD_TRY(expr)            \
  do {                           \
    int s_ = (expr);             \
    if (s_ != SSD_OK) return s_; \
  } while (0)

#define SSD_CHECK_ARG(cond, ...)      \
  do {                                \
    if (!(cond)) {                    \
      ::ssd::set_error(__VA_ARGS__);  \
      return SSD_EINVAL;              \
    }                                 \
  } while (0)

typedef uint16_t bf16_t;  // bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even; NaN stays NaN
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Activations between kernels.  fp32 models: plain fp32 [rows][cols].  bf16 models: two bf16 planes of the same
// shape, `plane` elements apart: head = bf16(x) and remainder = bf16(x - head), so that x = head + remainder to
// about 2^-17 relative and each plane is directly an MFMA operand.
template <typename T> struct Act;
template <> struct Act<float> {
  static __device__ __forceinline__ void store(void* base, int64_t plane, int64_t idx, float v) {
    (void)plane;
    ((float*)base)[idx] = v;
  }
};
template <> struct Act<bf16_t> {
  static __device__ __forceinline__ void store(void* base, int64_t plane, int64_t idx, float v) {
    bf16_t h = f32_to_bf16(v);
    ((bf16_t*)base)[idx] = h;
    ((bf16_t*)base)[plane + idx] = f32_to_bf16(v - bf16_to_f32(h));
  }
};

// One row of a batched forward pass (a branch at some depth, or one token of an extend).
struct RowDesc {
  int32_t seq;        // sequence b
  int32_t pos;        // absolute position of the row's token (rotary angle)
  int32_t vis;        // number of trunk positions the row sees (for extend rows this includes itself)
  int32_t suffix_len; // number of private suffix positions the row sees (includes itself); 0 for extend rows
  int32_t kv_slot;    // where the row's own K/V goes: trunk position (extend) or suffix depth (branch)
  int32_t is_branch;  // 1: KV goes to the row's private suffix, 0: to the trunk
};

// Shapes every kernel launcher needs.
struct Dims {
  int n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int dtype;
  float rope_theta, rms_eps;
  int q_dim() const { return n_q_heads * head_dim; }
  int kv_dim() const { return n_kv_heads * head_dim; }
  int qkv_dim() const { return q_dim() + 2 * kv_dim(); }
};

// Cache shape (Sec. 4.1.2): fan-out per accept length as running offsets.  Accept length k owns the F_k =
// off[k+1] - off[k] consecutive branch rows off[k] .. off[k+1]-1 of its sequence; off[K+1] is the rows per sequence.
// The uniform shape is off[k] = k F.  Passed to kernels by value.
struct FanTable {
  int32_t off[SSD_MAX_K + 2];
};

// ---------------------------------------------------------------- kernels_misc.hip
// Row descriptors + rotary tables for a branch step / an extend, from device-side trunk lengths.  The branch version
// also gathers the token every row feeds at this step into step_tokens (null: skipped).
int launch_setup_branch_rows(RowDesc* rows, float* cos_sin, const int32_t* trunk_len, int B, int K, const FanTable& fan, int step,
                             int half_dim, float theta, int32_t* step_tokens, const int32_t* keys,
                             const int32_t* cache_tokens, const int32_t* forced_keys, const int32_t* forced_tokens,
                             hipStream_t s);
int launch_setup_extend_rows(RowDesc* rows, float* cos_sin, const int32_t* trunk_len, int B, int T, int offset,
                             int half_dim, float theta, int seq_base, hipStream_t s);
int launch_embed(int dtype, const void* embed, const int32_t* tokens, float* h, int M, int d, int vocab, hipStream_t s);
int launch_rmsnorm(int dtype, const float* h, const void* gain, void* xn, int64_t xn_plane, float* copy_out,
                   int64_t copy_ld, int M, int d, float eps, hipStream_t s);
// Rotary embedding of q and k (fp32 [M][qkv_dim]) + write of q (activation dtype) and of the row's K/V
// into the trunk or its private suffix.
int launch_rope_append(int dtype, const float* qkv, const RowDesc* rows, const float* cos_sin, float* q_out,
                       void* trunk_k, void* trunk_v, void* suffix_k, void* suffix_v, int M, int n_q_heads,
                       int n_kv_heads, int head_dim, int max_trunk, int suffix_cap, hipStream_t s);
int launch_fill_i32(int32_t* p, int32_t v, int64_t n, hipStream_t s);
int launch_commit(int32_t* trunk_len, const int32_t* accept_len, int B, int K, hipStream_t s);
int launch_lookup(const int32_t* keys, const int32_t* cache_tokens, const float* cache_logits, const int32_t* accept_len,
                  const int32_t* bonus, uint8_t* hit, int32_t* branch, int32_t* spec, const float** logits_ptr, int B,
                  int K, const FanTable& fan, int V, hipStream_t s);
int launch_pending_exclude(int32_t* exclude, const int32_t* pending, int B, int K, hipStream_t s);
int launch_copy_kv_in(int dtype, void* trunk, const void* src, int B, int len, int max_trunk, int row_elems, hipStream_t s);

// ---------------------------------------------------------------- kernels_init.hip
// Seeded synthetic tensors generated on the device (bit-identical to the host-side input generators' twin).
// Tensor ids: 0 embedding, 1 LM head, 16 + 16 l + {0 wq, 1 wk, 2 wv, 3 wo, 4 w_gate, 5 w_up, 6 w_down} for layer l,
// 1 << 20 + 2 l + {0 keys, 1 values} for the synthetic prefix KV of layer l.
int launch_fill_hashed(int dtype, void* dst, int64_t n, uint64_t seed, uint64_t tensor_id, double std, hipStream_t s);
int launch_fill_const(int dtype, void* dst, int64_t n, float v, hipStream_t s);
int launch_fill_kv(int dtype, void* k, void* v, const int32_t* len, int B, int max_len, int Hkv, int D, int stride, int fused,
                   const int32_t* pages, int page_stride, uint64_t seed, uint64_t id_k, uint64_t id_v, hipStream_t s);

// ---------------------------------------------------------------- kernels_gemm.hip
enum GemmEpilogue { EPI_STORE_F32 = 0, EPI_RESIDUAL_ADD = 1, EPI_SWIGLU = 2 };
// Tiled copy of a [N][Kd] bf16 matrix into the MFMA-operand order the bf16 GEMM streams (see kernels_gemm.hip).
int launch_tile_weights_bf16(const bf16_t* src, bf16_t* dst, int N, int Kd, hipStream_t s);
// y[m][n] (+)= sum_k x[m][k] w[n][k].  x: activation [M][Kd] (planes `x_plane` apart for bf16 models); out fp32
// (ld elements); for EPI_SWIGLU out is an activation [M][N] = silu(x.w^T) * (x.w2^T) (planes `out_plane` apart).
int launch_gemm(int dtype, int epi, const void* x, int64_t x_plane, const void* w, const void* w2, void* out, int64_t ld,
                int64_t out_plane, int M, int N, int Kd, hipStream_t s);

// ---------------------------------------------------------------- kernels_attn.hip
struct AttnArgs {
  const float* q;        // fp32 [M][Hq][D]
  const void* trunk_k;   // model dtype [B][max_trunk][Hkv][D]
  const void* trunk_v;
  const void* suffix_k;  // model dtype [M][suffix_cap][Hkv][D]
  const void* suffix_v;
  void* out;             // activation [M][Hq][D]
  int64_t out_plane;
  const RowDesc* rows;
  float* partial;        // scratch for the partial softmaxes of key splits
  int64_t partial_floats;
  int M, n_q_heads, n_kv_heads, head_dim, max_trunk, suffix_cap;
  int rows_per_seq;      // rows of one sequence are consecutive
  int max_vis;           // host upper bound of any row's visible trunk length (grid sizing only)
};
int launch_attention(int dtype, const AttnArgs& a, hipStream_t s);
int64_t attention_partial_floats(int M, int n_q_heads, int head_dim, int max_keys);

// ---------------------------------------------------------------- kernels_select.hip
// scratch: top_f_scratch_bytes(rows) of device memory lets several blocks share a row (few rows of a large
// vocabulary would otherwise occupy a handful of compute units); null: one block per row.
int launch_top_f(const float* logits, int64_t ld, const int32_t* exclude, int rows, int V, int F, int32_t* ids,
                 void* scratch, hipStream_t s);
// The fan-out of a round: row (b, k) of logits [B (K+1)] gives its top F_k to ids[b][off[k] ..].
int launch_top_f_fan(const float* logits, int64_t ld, const int32_t* exclude, int B, int K, const FanTable& fan, int V,
                     int32_t* ids, void* scratch, hipStream_t s);
size_t top_f_scratch_bytes(int rows);
int launch_sample(const float* logits, int64_t ld, const float* temperature, int rows_per_seq, int rows, int V,
                  uint64_t seed, int row_base, int step, int32_t* out, int64_t out_stride, void* scratch, int exact_scan,
                  hipStream_t s);
size_t sample_scratch_bytes(int rows);
int launch_sigma_shift(float* logits, int64_t ld, const float* temperature, int rows_per_seq, int rows, int F,
                       const int32_t* ids, float log_c, hipStream_t s);
int launch_backup_random(int32_t* tokens, int B, int K, int V, uint64_t seed, hipStream_t s);
int launch_verify(const float* zt, const float* zd, const int32_t* spec, const float* temperature, int B, int K, int V,
                  uint64_t seed, int32_t* accept_len, int32_t* bonus, void* workspace, hipStream_t s);
size_t verify_workspace_bytes(int B, int K);
// the same with the workspace in a static device array of verify_static_capacity() bytes (no allocation, ever)
int launch_verify_static(const float* zt, const float* zd, const int32_t* spec, const float* temperature, int B, int K, int V,
                         uint64_t seed, int32_t* accept_len, int32_t* bonus, hipStream_t s);
size_t verify_static_capacity();

}  // namespace ssd
