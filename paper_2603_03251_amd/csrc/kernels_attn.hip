// Decode attention over "shared trunk + private suffix" (App. B: every branch row attends the verified trunk
// up to its fork point and only its own path).  No mask is materialised: a row is described by the number of
// trunk positions it sees and the number of private suffix positions it sees.
#include "common.h"

namespace ssd {

namespace {

template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const float* p, float* o) {
    float4 v = *(const float4*)p;
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const bf16_t* p, float* o) {
    uint4 v = *(const uint4*)p;
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

// One block per (row, KV head); wavefront w takes query heads w, w+4, .. of the group.  Each lane owns the keys
// lane, lane+64, .. and keeps its own running softmax (max, sum, weighted V); lanes are merged at the end.  The
// kernel for passes with many rows (every row is a block of its own, the chip is full without splitting keys).
template <typename T, int D>
__global__ __launch_bounds__(256) void attention_rowwise_kernel(const float* __restrict__ q, const T* __restrict__ trunk_k,
                                                                 const T* __restrict__ trunk_v,
                                                                 const T* __restrict__ suffix_k,
                                                                 const T* __restrict__ suffix_v, void* __restrict__ out,
                                                                 int64_t out_plane,
                                                                 const RowDesc* __restrict__ rows, int n_q_heads,
                                                                 int n_kv_heads, int max_trunk, int suffix_cap) {
  __shared__ float q_s[4][D];
  const int m = blockIdx.x, hk = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int group = n_q_heads / n_kv_heads;
  const RowDesc r = rows[m];
  const int n_keys = r.vis + r.suffix_len;
  const float scale = rsqrtf((float)D);
  const int64_t kv_stride = (int64_t)n_kv_heads * D;
  const T* tk = trunk_k + ((int64_t)r.seq * max_trunk) * kv_stride + hk * D;
  const T* tv = trunk_v + ((int64_t)r.seq * max_trunk) * kv_stride + hk * D;
  const T* sk = suffix_k + ((int64_t)m * suffix_cap) * kv_stride + hk * D;
  const T* sv = suffix_v + ((int64_t)m * suffix_cap) * kv_stride + hk * D;

  for (int g = wave; g < group; g += 4) {
    const int hq = hk * group + g;
    const float* qp = q + ((int64_t)m * n_q_heads + hq) * D;
    for (int d = lane; d < D; d += 64) q_s[wave][d] = qp[d];
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

    float m_run = -INFINITY, l_run = 0.f;
    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;

    for (int j = lane; j < n_keys; j += 64) {
      const T* kp = j < r.vis ? tk + (int64_t)j * kv_stride : sk + (int64_t)(j - r.vis) * kv_stride;
      const T* vp = j < r.vis ? tv + (int64_t)j * kv_stride : sv + (int64_t)(j - r.vis) * kv_stride;
      float s = 0.f;
#pragma unroll
      for (int d0 = 0; d0 < D; d0 += Vec16<T>::N) {
        float kk[Vec16<T>::N];
        Vec16<T>::load(kp + d0, kk);
#pragma unroll
        for (int e = 0; e < Vec16<T>::N; ++e) s = fmaf(q_s[wave][d0 + e], kk[e], s);
      }
      s *= scale;
      float m_new = fmaxf(m_run, s);
      float corr = expf(m_run - m_new);      // exp(-inf) = 0 on the first key
      float p = expf(s - m_new);
      l_run = l_run * corr + p;
#pragma unroll
      for (int d0 = 0; d0 < D; d0 += Vec16<T>::N) {
        float vv[Vec16<T>::N];
        Vec16<T>::load(vp + d0, vv);
#pragma unroll
        for (int e = 0; e < Vec16<T>::N; ++e) acc[d0 + e] = fmaf(p, vv[e], acc[d0 + e] * corr);
      }
      m_run = m_new;
    }
    // merge the 64 lanes
    float m_all = m_run;
    for (int o = 32; o > 0; o >>= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, o));
    float w = m_run == -INFINITY ? 0.f : expf(m_run - m_all);
    float l_all = l_run * w;
    for (int o = 32; o > 0; o >>= 1) l_all += __shfl_xor(l_all, o);
    float inv = 1.0f / l_all;
    const int64_t obase = ((int64_t)m * n_q_heads + hq) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) {
      float v = acc[d] * w;
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
      if (lane == (d & 63)) Act<T>::store(out, out_plane, obase + d, v * inv);
    }
    __builtin_amdgcn_wave_barrier();
  }
}

constexpr int kMaxSplits = 64;          // key splits of a row
constexpr int kSplitKeys = 256;         // most keys of a split: one per thread
constexpr int kSplitMaxRows = 64;       // rows up to which the scratch allows the most splits
constexpr int kSplitMaxGroup = 8;       // query heads per KV head the split kernel holds

template <typename T, int NE> struct LoadElems;
template <> struct LoadElems<bf16_t, 1> { static __device__ __forceinline__ void load(const bf16_t* p, float* o) { o[0] = bf16_to_f32(p[0]); } };
template <> struct LoadElems<bf16_t, 2> {
  static __device__ __forceinline__ void load(const bf16_t* p, float* o) {
    const uint32_t w = *(const uint32_t*)p;
    o[0] = __uint_as_float(w << 16);
    o[1] = __uint_as_float(w & 0xffff0000u);
  }
};
template <> struct LoadElems<float, 1> { static __device__ __forceinline__ void load(const float* p, float* o) { o[0] = p[0]; } };
template <> struct LoadElems<float, 2> {
  static __device__ __forceinline__ void load(const float* p, float* o) {
    const float2 v = *(const float2*)p;
    o[0] = v.x;
    o[1] = v.y;
  }
};

// Passes with few rows (an extend, a verification forward, a small decode batch): one block per (row, KV head, split
// of at most 256 keys), all query heads of the group at once.  Scores: one key per thread against the group's queries
// (in LDS); softmax over the block; weighted values: thread = (quarter of the keys, D/64 head dimensions), so every
// value row is read with consecutive threads on consecutive dimensions.  Writes the split's partial softmax
// (max, sum, unnormalised output) to `partial` [row][query head][split][D + 2]; attention_merge_kernel adds the
// splits up in split order.
template <typename T, int D>
__global__ __launch_bounds__(256) void attention_split_kernel(const float* __restrict__ q, const T* __restrict__ trunk_k,
                                                               const T* __restrict__ trunk_v, const T* __restrict__ suffix_k,
                                                               const T* __restrict__ suffix_v, const RowDesc* __restrict__ rows,
                                                               int n_q_heads, int n_kv_heads, int max_trunk, int suffix_cap,
                                                               float* __restrict__ partial, int keys_per_split) {
  constexpr int G = kSplitMaxGroup, NE = D / 64;
  __shared__ float q_s[G][D];
  __shared__ float p_s[G][kSplitKeys];
  __shared__ float red_s[4][G][D];
  __shared__ float mx_s[G][4], sum_s[G][4];
  const int m = blockIdx.x, hk = blockIdx.y, split = blockIdx.z, n_splits = gridDim.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int group = n_q_heads / n_kv_heads;
  const RowDesc r = rows[m];
  const int n_keys = r.vis + r.suffix_len;
  const int j_begin = split * keys_per_split;
  const int j_end = min(n_keys, j_begin + keys_per_split);
  const float scale = rsqrtf((float)D);
  const int64_t kv_stride = (int64_t)n_kv_heads * D;
  const T* tk = trunk_k + ((int64_t)r.seq * max_trunk) * kv_stride + hk * D;
  const T* tv = trunk_v + ((int64_t)r.seq * max_trunk) * kv_stride + hk * D;
  const T* sk = suffix_k + ((int64_t)m * suffix_cap) * kv_stride + hk * D;
  const T* sv = suffix_v + ((int64_t)m * suffix_cap) * kv_stride + hk * D;

  for (int i = tid; i < group * D; i += 256) {
    const int g = i / D, d = i - g * D;
    q_s[g][d] = q[((int64_t)m * n_q_heads + hk * group + g) * D + d] * scale;
  }
  __syncthreads();

  // ---- scores of key j_begin + tid against the group's queries
  const int j = j_begin + tid;
  const bool have = j < j_end;
  float sc[G];
#pragma unroll
  for (int g = 0; g < G; ++g) sc[g] = 0.f;
  if (have) {
    const T* kp = j < r.vis ? tk + (int64_t)j * kv_stride : sk + (int64_t)(j - r.vis) * kv_stride;
    // (fully unrolled: the key row's loads all go out before the first product; in groups of 4 a row of 128 bf16
    // cost four memory round trips)
#pragma unroll
    for (int d0 = 0; d0 < D; d0 += Vec16<T>::N) {
      float kk[Vec16<T>::N];
      Vec16<T>::load(kp + d0, kk);
#pragma unroll
      for (int g = 0; g < G; ++g)
        if (g < group) {
#pragma unroll
          for (int e = 0; e < Vec16<T>::N; ++e) sc[g] = fmaf(q_s[g][d0 + e], kk[e], sc[g]);
        }
    }
  }
  // ---- softmax over the split: maximum and sum per query head
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float v = have ? sc[g] : -INFINITY;
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    if (lane == 0) mx_s[g][wave] = v;
  }
  __syncthreads();
  float mg[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    mg[g] = fmaxf(fmaxf(mx_s[g][0], mx_s[g][1]), fmaxf(mx_s[g][2], mx_s[g][3]));
    const float m_use = mg[g] == -INFINITY ? 0.f : mg[g];
    const float pe = have ? expf(sc[g] - m_use) : 0.f;
    p_s[g][tid] = pe;
    float v = pe;
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if (lane == 0) sum_s[g][wave] = v;
  }
  __syncthreads();
  // ---- weighted values: wavefront = quarter of the split's keys, lane = NE consecutive head dimensions
  float acc[G][NE];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < NE; ++e) acc[g][e] = 0.f;
  const int jq0 = wave * (kSplitKeys / 4);
  const int jq1 = min(jq0 + kSplitKeys / 4, j_end - j_begin);
  // value rows in batches of kPvBatch whose loads go out together (one row per iteration, used at once, made the loop
  // a chain of memory latencies: 64 of them per wavefront); rows past the quarter's end re-read its last row
  constexpr int kPvBatch = 8;
  for (int jj0 = jq0; jj0 < jq1; jj0 += kPvBatch) {
    float vv[kPvBatch][NE];
#pragma unroll
    for (int u = 0; u < kPvBatch; ++u) {
      const int jk = j_begin + min(jj0 + u, jq1 - 1);
      const T* vp = (jk < r.vis ? tv + (int64_t)jk * kv_stride : sv + (int64_t)(jk - r.vis) * kv_stride) + lane * NE;
      LoadElems<T, NE>::load(vp, vv[u]);
    }
#pragma unroll
    for (int u = 0; u < kPvBatch; ++u) {
      if (jj0 + u < jq1) {
#pragma unroll
        for (int g = 0; g < G; ++g)
          if (g < group) {
            const float pe = p_s[g][jj0 + u];
#pragma unroll
            for (int e = 0; e < NE; ++e) acc[g][e] = fmaf(pe, vv[u][e], acc[g][e]);
          }
      }
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int e = 0; e < NE; ++e) red_s[wave][g][lane * NE + e] = acc[g][e];
  __syncthreads();
  for (int i = tid; i < group * D; i += 256) {
    const int g = i / D, d = i - g * D;
    float* pp = partial + (((int64_t)m * n_q_heads + hk * group + g) * n_splits + split) * (D + 2);
    pp[2 + d] = (red_s[0][g][d] + red_s[1][g][d]) + (red_s[2][g][d] + red_s[3][g][d]);
    if (d == 0) {
      pp[0] = fmaxf(fmaxf(mx_s[g][0], mx_s[g][1]), fmaxf(mx_s[g][2], mx_s[g][3]));   // -inf for a split without keys
      pp[1] = (sum_s[g][0] + sum_s[g][1]) + (sum_s[g][2] + sum_s[g][3]);
    }
  }
}

// One block per (row, query head), one thread per head dimension: the splits' partial softmaxes in split order.
template <typename T, int D>
__global__ __launch_bounds__(D) void attention_merge_kernel(const float* __restrict__ partial, void* __restrict__ out,
                                                            int64_t out_plane, int n_splits) {
  const int64_t pair = blockIdx.x;
  const int d = threadIdx.x;
  const float* pp = partial + pair * n_splits * (D + 2);
  float m_max = -INFINITY;
#pragma unroll 8
  for (int s = 0; s < n_splits; ++s) m_max = fmaxf(m_max, pp[s * (D + 2)]);
  float l = 0.f, o = 0.f;
#pragma unroll 8
  for (int s = 0; s < n_splits; ++s) {
    const float ms = pp[s * (D + 2)];
    const float w = ms == -INFINITY ? 0.f : expf(ms - m_max);
    l += w * pp[s * (D + 2) + 1];
    o += w * pp[s * (D + 2) + 2 + d];
  }
  Act<T>::store(out, out_plane, pair * D + d, o / l);
}

// Splits of at most kSplitKeys keys, and with few rows enough of them for about 1024 blocks (none shorter than 64
// keys); 1 (the row-wise kernel) when the shape is outside what the split kernel holds or the scratch is too small.
int choose_splits(const AttnArgs& a, int* keys_per_split) {
  const int pairs = a.M * a.n_kv_heads;
  const int max_keys = (a.max_vis > 0 ? a.max_vis : 0) + a.suffix_cap;
  *keys_per_split = 0;
  if (!a.partial || a.n_q_heads / a.n_kv_heads > kSplitMaxGroup) return 1;
  int n = (max_keys + kSplitKeys - 1) / kSplitKeys;
  int fill = (1024 + pairs - 1) / pairs;
  const int by_len = (max_keys + 63) / 64;
  fill = fill < by_len ? fill : by_len;
  n = n > fill ? n : fill;
  if (n < 1) n = 1;
  if (n > kMaxSplits || (int64_t)a.M * a.n_q_heads * n * (a.head_dim + 2) > a.partial_floats) return 1;
  *keys_per_split = ((max_keys + n - 1) / n + 63) / 64 * 64;
  return n;
}

template <typename T, int D>
int launch_rowwise_d(const AttnArgs& a, hipStream_t s) {
  int keys_per_split = 0;
  const int n_splits = choose_splits(a, &keys_per_split);
  if (keys_per_split == 0) {
    dim3 grid(a.M, a.n_kv_heads);
    attention_rowwise_kernel<T, D><<<grid, 256, 0, s>>>(a.q, (const T*)a.trunk_k, (const T*)a.trunk_v, (const T*)a.suffix_k,
                                                        (const T*)a.suffix_v, a.out, a.out_plane, a.rows, a.n_q_heads,
                                                        a.n_kv_heads, a.max_trunk, a.suffix_cap);
  } else {
    dim3 grid(a.M, a.n_kv_heads, n_splits);
    attention_split_kernel<T, D><<<grid, 256, 0, s>>>(a.q, (const T*)a.trunk_k, (const T*)a.trunk_v, (const T*)a.suffix_k,
                                                      (const T*)a.suffix_v, a.rows, a.n_q_heads, a.n_kv_heads, a.max_trunk,
                                                      a.suffix_cap, a.partial, keys_per_split);
    SSD_HIP(hipGetLastError());
    attention_merge_kernel<T, D><<<a.M * a.n_q_heads, D, 0, s>>>(a.partial, a.out, a.out_plane, n_splits);
  }
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

template <typename T>
int launch_rowwise(const AttnArgs& a, hipStream_t s) {
  if (a.head_dim == 64) return launch_rowwise_d<T, 64>(a, s);
  if (a.head_dim == 128) return launch_rowwise_d<T, 128>(a, s);
  set_error("head_dim %d not supported (64 or 128)", a.head_dim);
  return SSD_EINVAL;
}

}  // namespace

// Floats of split-softmax scratch for contexts of up to M rows: few rows x many splits, or M rows x the splits that
// max_keys keys need.
int64_t attention_partial_floats(int M, int n_q_heads, int head_dim, int max_keys) {
  const int64_t few = (int64_t)(M < kSplitMaxRows ? M : kSplitMaxRows) * kMaxSplits;
  const int64_t many = (int64_t)M * ((max_keys + kSplitKeys - 1) / kSplitKeys + 1);
  return (few > many ? few : many) * n_q_heads * (head_dim + 2);
}

int launch_attention(int dtype, const AttnArgs& a, hipStream_t s) {
  if (a.M <= 0) return SSD_OK;
  return dtype == SSD_BF16 ? launch_rowwise<bf16_t>(a, s) : launch_rowwise<float>(a, s);
}

}  // namespace ssd
