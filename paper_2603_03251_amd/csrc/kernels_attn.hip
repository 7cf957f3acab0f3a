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
// lane, lane+64, .. and keeps its own running softmax (max, sum, weighted V); lanes are merged at the end.
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

template <typename T>
int launch_rowwise(const AttnArgs& a, hipStream_t s) {
  dim3 grid(a.M, a.n_kv_heads);
  if (a.head_dim == 64)
    attention_rowwise_kernel<T, 64><<<grid, 256, 0, s>>>(a.q, (const T*)a.trunk_k, (const T*)a.trunk_v,
                                                         (const T*)a.suffix_k, (const T*)a.suffix_v, a.out, a.out_plane, a.rows,
                                                         a.n_q_heads, a.n_kv_heads, a.max_trunk, a.suffix_cap);
  else if (a.head_dim == 128)
    attention_rowwise_kernel<T, 128><<<grid, 256, 0, s>>>(a.q, (const T*)a.trunk_k, (const T*)a.trunk_v,
                                                          (const T*)a.suffix_k, (const T*)a.suffix_v, a.out, a.out_plane, a.rows,
                                                          a.n_q_heads, a.n_kv_heads, a.max_trunk, a.suffix_cap);
  else {
    set_error("head_dim %d not supported (64 or 128)", a.head_dim);
    return SSD_EINVAL;
  }
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

}  // namespace

size_t attention_partial_bytes(int M, int n_q_heads, int head_dim, int max_trunk) {
  (void)M; (void)n_q_heads; (void)head_dim; (void)max_trunk;
  return 256;
}

int launch_attention(int dtype, const AttnArgs& a, hipStream_t s) {
  if (a.M <= 0) return SSD_OK;
  return dtype == SSD_BF16 ? launch_rowwise<bf16_t>(a, s) : launch_rowwise<float>(a, s);
}

}  // namespace ssd
