// Small kernels of the round: row descriptors and rotary tables, embedding gather, RMSNorm,
// rotary embedding + KV append, step-token gather, cache lookup, trunk commit.
#include "common.h"

namespace ssd {

namespace {

constexpr int kBlock = 256;

// Rotary table entry for (row, i): cos and sin of pos * theta^(-2i/D), evaluated in fp64.
__device__ __forceinline__ void write_cos_sin(float* cos_sin, int row, int half_dim, int i, int pos, float theta) {
  double inv = pow((double)theta, -2.0 * (double)i / (double)(2 * half_dim));
  double ang = (double)pos * inv;
  cos_sin[((int64_t)row * half_dim + i) * 2 + 0] = (float)cos(ang);
  cos_sin[((int64_t)row * half_dim + i) * 2 + 1] = (float)sin(ang);
}

// Branch rows at depth `step` (App. B): row (b,k,j) sits at position trunk_len+1+k+step, sees the trunk up to
// the glue position of accept length k, and its own step+1 private positions.
// Everything a branch-decode step needs before its forward pass, in one launch: the row descriptors and rotary tables
// of step `step`, and the token every row feeds (its cache key at step 0, afterwards the token it drew one step
// earlier; the forced arrays replace both under teacher forcing).
__global__ void setup_branch_rows_kernel(RowDesc* rows, float* cos_sin, const int32_t* trunk_len, int M, int K,
                                         FanTable fan, int step, int half_dim, float theta, int32_t* step_tokens, const int32_t* keys,
                                         const int32_t* cache_tokens, const int32_t* forced_keys,
                                         const int32_t* forced_tokens) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= M * half_dim) return;
  int m = idx / half_dim, i = idx % half_dim;
  const int per_seq = fan.off[K + 1];
  int b = m / per_seq, within = m - b * per_seq;
  int k = 0;
  while (k < K && within >= fan.off[k + 1]) ++k;
  int tl = trunk_len[b];
  int pos = tl + 1 + k + step;
  if (i == 0) {
    RowDesc r;
    r.seq = b; r.pos = pos; r.vis = tl + k + 1; r.suffix_len = step + 1; r.kv_slot = step; r.is_branch = 1;
    rows[m] = r;
    if (step_tokens) {
      if (step == 0) step_tokens[m] = forced_keys ? forced_keys[m] : keys[m];
      else step_tokens[m] = forced_tokens ? forced_tokens[(int64_t)m * K + step - 1] : cache_tokens[(int64_t)m * K + step - 1];
    }
  }
  write_cos_sin(cos_sin, m, half_dim, i, pos, theta);
}

// Extend rows: token t of sequence b at position trunk_len+offset+t, causal (sees itself after the append).
// rows of sequences seq_base .. seq_base + B - 1 (row m of the pass = token m % T of sequence seq_base + m / T)
__global__ void setup_extend_rows_kernel(RowDesc* rows, float* cos_sin, const int32_t* trunk_len, int B, int T,
                                         int offset, int half_dim, float theta, int seq_base) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * T * half_dim) return;
  int m = idx / half_dim, i = idx % half_dim;
  int b = seq_base + m / T, t = m % T;
  int pos = trunk_len[b] + offset + t;
  if (i == 0) {
    RowDesc r;
    r.seq = b; r.pos = pos; r.vis = pos + 1; r.suffix_len = 0; r.kv_slot = pos; r.is_branch = 0;
    rows[m] = r;
  }
  write_cos_sin(cos_sin, m, half_dim, i, pos, theta);
}

template <typename T>
__global__ void embed_kernel(const T* embed, const int32_t* tokens, float* h, int M, int d, int vocab) {
  int m = blockIdx.x;
  int tok = tokens[m];
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
  const T* src = embed + (int64_t)tok * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) h[(int64_t)m * d + c] = Elem<T>::load(src + c);
}

__device__ __forceinline__ float block_sum(float v, float* smem) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  if ((threadIdx.x & 63) == 0) smem[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += smem[i];
  __syncthreads();
  return t;
}

// x / sqrt(mean(x^2) + eps) * gain, one block per row.  The row is read once, four elements per thread and step,
// with the loads of up to 8 steps issued together (a row of 8192 is then one memory latency, not 32).
template <typename T>
__global__ void rmsnorm_kernel(const float* __restrict__ h, const T* __restrict__ gain, void* __restrict__ xn, int64_t xn_plane,
                               float* __restrict__ copy_out, int64_t copy_ld, int d, float eps) {
  __shared__ float smem[kBlock / 64];
  const int m = blockIdx.x;
  const float* row = h + (int64_t)m * d;
  constexpr int kHeld = 8;                      // float4 per thread kept in registers
  const int step = blockDim.x * 4;
  float4 held[kHeld];
  uint2 gheld[kHeld];                           // bf16 gains of the held elements, requested with them
  float ss = 0.f;
  const bool vec = (d & 3) == 0;
  const bool aligned = (xn_plane & 3) == 0 && (copy_ld & 3) == 0 && ((uintptr_t)xn & 7) == 0 && ((uintptr_t)gain & 7) == 0 &&
                       (!copy_out || ((uintptr_t)copy_out & 15) == 0);
  if (vec) {
#pragma unroll
    for (int i = 0; i < kHeld; ++i) {
      const int c = threadIdx.x * 4 + i * step;
      held[i] = c < d ? *(const float4*)(row + c) : make_float4(0.f, 0.f, 0.f, 0.f);
      if constexpr (sizeof(T) == 2) gheld[i] = (aligned && c < d) ? *(const uint2*)((const bf16_t*)gain + c) : make_uint2(0u, 0u);
    }
#pragma unroll
    for (int i = 0; i < kHeld; ++i) ss += held[i].x * held[i].x + held[i].y * held[i].y + held[i].z * held[i].z + held[i].w * held[i].w;
    for (int c = threadIdx.x + kHeld * step; c < d; c += blockDim.x) { float v = row[c]; ss += v * v; }
  } else {
    for (int c = threadIdx.x; c < d; c += blockDim.x) { float v = row[c]; ss += v * v; }
  }
  ss = block_sum(ss, smem);
  const float scale = 1.0f / sqrtf(ss / (float)d + eps);
  auto put = [&](int c, float x) {
    const float v = x * scale * Elem<T>::load(gain + c);
    Act<T>::store(xn, xn_plane, (int64_t)m * d + c, v);
    if (copy_out) copy_out[(int64_t)m * copy_ld + c] = v;
  };
  if (vec) {
    // four features at a time: one 8-byte gain load, one 8-byte store per bf16 plane (2-byte stores, one per element
    // and plane, made this kernel several times slower than the memory round trips it consists of)
    auto put4 = [&](int c, float4 x, uint2 gb) {
      if constexpr (sizeof(T) == 2) {
        const float g[4] = {__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xffff0000u), __uint_as_float(gb.y << 16),
                            __uint_as_float(gb.y & 0xffff0000u)};
        const float v[4] = {x.x * scale * g[0], x.y * scale * g[1], x.z * scale * g[2], x.w * scale * g[3]};
        bf16_t hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          hi[e] = f32_to_bf16(v[e]);
          lo[e] = f32_to_bf16(v[e] - bf16_to_f32(hi[e]));
        }
        bf16_t* base = (bf16_t*)xn + (int64_t)m * d + c;
        *(uint2*)base = make_uint2((uint32_t)hi[0] | (uint32_t)hi[1] << 16, (uint32_t)hi[2] | (uint32_t)hi[3] << 16);
        *(uint2*)(base + xn_plane) = make_uint2((uint32_t)lo[0] | (uint32_t)lo[1] << 16, (uint32_t)lo[2] | (uint32_t)lo[3] << 16);
        if (copy_out) *(float4*)(copy_out + (int64_t)m * copy_ld + c) = make_float4(v[0], v[1], v[2], v[3]);
      } else {
        put(c, x.x);
        put(c + 1, x.y);
        put(c + 2, x.z);
        put(c + 3, x.w);
      }
    };
#pragma unroll
    for (int i = 0; i < kHeld; ++i) {
      const int c = threadIdx.x * 4 + i * step;
      if (c < d) {
        if (aligned) put4(c, held[i], gheld[i]);
        else {
          put(c, held[i].x);
          put(c + 1, held[i].y);
          put(c + 2, held[i].z);
          put(c + 3, held[i].w);
        }
      }
    }
    for (int c = threadIdx.x + kHeld * step; c < d; c += blockDim.x) put(c, row[c]);
  } else {
    for (int c = threadIdx.x; c < d; c += blockDim.x) put(c, row[c]);
  }
}

// Rotary embedding (pair (i, i + D/2)) of the q and k heads of one row; q goes out in the activation type,
// k and v go to the row's KV slot (trunk position or private suffix depth).
template <typename T>
__global__ void rope_append_kernel(const float* __restrict__ qkv, const RowDesc* __restrict__ rows, const float* __restrict__ cos_sin,
                                   float* __restrict__ q_out, T* __restrict__ trunk_k, T* __restrict__ trunk_v,
                                   T* __restrict__ suffix_k, T* __restrict__ suffix_v, int n_q_heads, int n_kv_heads, int head_dim,
                                   int max_trunk, int suffix_cap) {
  int m = blockIdx.x;
  RowDesc r = rows[m];
  int half = head_dim >> 1;
  int qd = n_q_heads * head_dim, kvd = n_kv_heads * head_dim;
  const float* src = qkv + (int64_t)m * (qd + 2 * kvd);
  int64_t kv_row = r.is_branch ? ((int64_t)m * suffix_cap + r.kv_slot) : ((int64_t)r.seq * max_trunk + r.kv_slot);
  T* kdst = (r.is_branch ? suffix_k : trunk_k) + kv_row * kvd;
  T* vdst = (r.is_branch ? suffix_v : trunk_v) + kv_row * kvd;
  const float* cs = cos_sin + (int64_t)m * half * 2;
  int n_rot = (n_q_heads + n_kv_heads) * half;
  // items in batches whose loads go out together (a 70B-shaped row has 18 items per thread: one at a time they were 18
  // memory round trips); the input and the outputs never overlap, which the qualifiers above tell the compiler
  constexpr int kBatch = 6;
  for (int idx0 = threadIdx.x; idx0 < n_rot; idx0 += blockDim.x * kBatch) {
    float a[kBatch], b[kBatch], c[kBatch], sn[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int idx = min(idx0 + u * (int)blockDim.x, n_rot - 1);
      const int head = idx / half, i = idx % half;
      const float* hsrc = src + head * head_dim;   // q heads then k heads are contiguous in qkv
      c[u] = cs[i * 2];
      sn[u] = cs[i * 2 + 1];
      a[u] = hsrc[i];
      b[u] = hsrc[i + half];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int idx = idx0 + u * (int)blockDim.x;
      if (idx >= n_rot) break;
      const int head = idx / half, i = idx % half;
      const float ra = a[u] * c[u] - b[u] * sn[u], rb = b[u] * c[u] + a[u] * sn[u];
      if (head < n_q_heads) {
        float* dst = q_out + (int64_t)m * qd + head * head_dim;
        dst[i] = ra;
        dst[i + half] = rb;
      } else {
        T* dst = kdst + (head - n_q_heads) * head_dim;
        Elem<T>::store(dst + i, ra);
        Elem<T>::store(dst + i + half, rb);
      }
    }
  }
  for (int c = threadIdx.x; c < kvd; c += blockDim.x) Elem<T>::store(vdst + c, src[qd + kvd + c]);
}

// p[0 .. n-1] = v
__global__ void fill_i32_kernel(int32_t* p, int32_t v, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void commit_kernel(int32_t* trunk_len, const int32_t* accept_len, int B, int K) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int k = accept_len[b];
  k = k < 0 ? 0 : (k > K ? K : k);
  trunk_len[b] += k + 1;
}

// One thread per sequence: linear scan of the F_k keys cached for accept length k.
__global__ void lookup_kernel(const int32_t* keys, const int32_t* cache_tokens, const float* cache_logits,
                              const int32_t* accept_len, const int32_t* bonus, uint8_t* hit, int32_t* branch,
                              int32_t* spec, const float** logits_ptr, int B, int K, FanTable fan, int V) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int k = accept_len[b], t = bonus[b], found = -1;
  int64_t first = 0;
  if (k >= 0 && k <= K) {
    first = (int64_t)b * fan.off[K + 1] + fan.off[k];
    const int F = fan.off[k + 1] - fan.off[k];
    for (int j = 0; j < F; ++j)
      if (keys[first + j] == t) { found = j; break; }
  }
  hit[b] = found >= 0 ? 1 : 0;
  branch[b] = found;
  int64_t m = first + found;
  for (int i = 0; i < K; ++i) spec[(int64_t)b * K + i] = found >= 0 ? cache_tokens[m * K + i] : -1;
  if (logits_ptr) logits_ptr[b] = found >= 0 ? cache_logits + m * (int64_t)K * V : nullptr;
}

// exclude[b][k] = s_{k+1} for k < K, -1 for k = K (Sec. 4.1.1: the token sent for verification is skipped).
__global__ void pending_exclude_kernel(int32_t* exclude, const int32_t* pending, int B, int K) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * (K + 1)) return;
  int b = idx / (K + 1), k = idx % (K + 1);
  exclude[idx] = k < K ? pending[(int64_t)b * (K + 1) + k + 1] : -1;
}

template <typename T>
__global__ void copy_kv_in_kernel(T* trunk, const T* src, int len, int max_trunk, int row_elems, int64_t total) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  int64_t per_seq = (int64_t)len * row_elems;
  int64_t b = idx / per_seq, rem = idx % per_seq;
  trunk[b * (int64_t)max_trunk * row_elems + rem] = src[idx];
}

inline int grid_for(int64_t n) { return (int)((n + kBlock - 1) / kBlock); }

}  // namespace

int launch_setup_branch_rows(RowDesc* rows, float* cos_sin, const int32_t* trunk_len, int B, int K, const FanTable& fan, int step,
                             int half_dim, float theta, int32_t* step_tokens, const int32_t* keys,
                             const int32_t* cache_tokens, const int32_t* forced_keys, const int32_t* forced_tokens,
                             hipStream_t s) {
  const int M = B * fan.off[K + 1];
  setup_branch_rows_kernel<<<grid_for((int64_t)M * half_dim), kBlock, 0, s>>>(rows, cos_sin, trunk_len, M, K, fan, step,
                                                                             half_dim, theta, step_tokens, keys,
                                                                             cache_tokens, forced_keys, forced_tokens);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_setup_extend_rows(RowDesc* rows, float* cos_sin, const int32_t* trunk_len, int B, int T, int offset,
                             int half_dim, float theta, int seq_base, hipStream_t s) {
  setup_extend_rows_kernel<<<grid_for((int64_t)B * T * half_dim), kBlock, 0, s>>>(rows, cos_sin, trunk_len, B, T,
                                                                                 offset, half_dim, theta, seq_base);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_embed(int dtype, const void* embed, const int32_t* tokens, float* h, int M, int d, int vocab, hipStream_t s) {
  if (dtype == SSD_BF16) embed_kernel<bf16_t><<<M, kBlock, 0, s>>>((const bf16_t*)embed, tokens, h, M, d, vocab);
  else embed_kernel<float><<<M, kBlock, 0, s>>>((const float*)embed, tokens, h, M, d, vocab);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_rmsnorm(int dtype, const float* h, const void* gain, void* xn, int64_t xn_plane, float* copy_out,
                   int64_t copy_ld, int M, int d, float eps, hipStream_t s) {
  if (dtype == SSD_BF16)
    rmsnorm_kernel<bf16_t><<<M, kBlock, 0, s>>>(h, (const bf16_t*)gain, xn, xn_plane, copy_out, copy_ld, d, eps);
  else
    rmsnorm_kernel<float><<<M, kBlock, 0, s>>>(h, (const float*)gain, xn, xn_plane, copy_out, copy_ld, d, eps);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_rope_append(int dtype, const float* qkv, const RowDesc* rows, const float* cos_sin, float* q_out,
                       void* trunk_k, void* trunk_v, void* suffix_k, void* suffix_v, int M, int n_q_heads,
                       int n_kv_heads, int head_dim, int max_trunk, int suffix_cap, hipStream_t s) {
  if (dtype == SSD_BF16)
    rope_append_kernel<bf16_t><<<M, kBlock, 0, s>>>(qkv, rows, cos_sin, q_out, (bf16_t*)trunk_k,
                                                    (bf16_t*)trunk_v, (bf16_t*)suffix_k, (bf16_t*)suffix_v, n_q_heads,
                                                    n_kv_heads, head_dim, max_trunk, suffix_cap);
  else
    rope_append_kernel<float><<<M, kBlock, 0, s>>>(qkv, rows, cos_sin, q_out, (float*)trunk_k, (float*)trunk_v,
                                                   (float*)suffix_k, (float*)suffix_v, n_q_heads, n_kv_heads, head_dim,
                                                   max_trunk, suffix_cap);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_fill_i32(int32_t* p, int32_t v, int64_t n, hipStream_t s) {
  if (n <= 0) return SSD_OK;
  fill_i32_kernel<<<grid_for(n), kBlock, 0, s>>>(p, v, n);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_commit(int32_t* trunk_len, const int32_t* accept_len, int B, int K, hipStream_t s) {
  commit_kernel<<<grid_for(B), kBlock, 0, s>>>(trunk_len, accept_len, B, K);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_lookup(const int32_t* keys, const int32_t* cache_tokens, const float* cache_logits, const int32_t* accept_len,
                  const int32_t* bonus, uint8_t* hit, int32_t* branch, int32_t* spec, const float** logits_ptr, int B,
                  int K, const FanTable& fan, int V, hipStream_t s) {
  lookup_kernel<<<grid_for(B), kBlock, 0, s>>>(keys, cache_tokens, cache_logits, accept_len, bonus, hit, branch, spec,
                                               logits_ptr, B, K, fan, V);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_pending_exclude(int32_t* exclude, const int32_t* pending, int B, int K, hipStream_t s) {
  pending_exclude_kernel<<<grid_for((int64_t)B * (K + 1)), kBlock, 0, s>>>(exclude, pending, B, K);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_copy_kv_in(int dtype, void* trunk, const void* src, int B, int len, int max_trunk, int row_elems,
                      hipStream_t s) {
  int64_t total = (int64_t)B * len * row_elems;
  if (total == 0) return SSD_OK;
  if (dtype == SSD_BF16)
    copy_kv_in_kernel<bf16_t><<<grid_for(total), kBlock, 0, s>>>((bf16_t*)trunk, (const bf16_t*)src, len, max_trunk,
                                                                row_elems, total);
  else
    copy_kv_in_kernel<float><<<grid_for(total), kBlock, 0, s>>>((float*)trunk, (const float*)src, len, max_trunk,
                                                               row_elems, total);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

}  // namespace ssd
