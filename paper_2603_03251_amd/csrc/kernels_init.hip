// Seeded synthetic content generated on the device: random-init weights and a synthetic prefix KV, so that a model of
// any size (the 70B-shaped target holds 139 GB of weights) exists without a host copy.  The values are defined by
// integer arithmetic only, so a host-side twin (the input generators of the tests) produces the same bits:
//   bits  = mix64(mix64(seed + GOLD * (tensor id + 1)) + element index)          (SplitMix64 finaliser)
//   S     = sum of the four 16-bit lanes of bits            (Irwin-Hall: mean 131070, standard deviation 37837.2...)
//   value = float(S - 131070) * scale, scale = float(std / 37837.227...) computed in double on the host,
// one exact int -> float conversion and one fp32 multiplication, then round-to-nearest-even to bf16 for bf16 tensors.
#include "common.h"
#include "rng.h"

namespace ssd {

namespace {

constexpr uint64_t kGold = 0x9E3779B97F4A7C15ull;
constexpr double kIrwinHallSigma = 37837.22723537048;   // sqrt(4 (65536^2 - 1) / 12)

__host__ __device__ __forceinline__ uint64_t tensor_prefix(uint64_t seed, uint64_t tensor_id) {
  return mix64(seed + kGold * (tensor_id + 1));
}
__device__ __forceinline__ float hashed_value(uint64_t prefix, uint64_t index, float scale) {
  const uint64_t b = mix64(prefix + index);
  const int s = (int)(b & 0xffff) + (int)((b >> 16) & 0xffff) + (int)((b >> 32) & 0xffff) + (int)(b >> 48);
  return (float)(s - 131070) * scale;
}

template <typename T>
__global__ void fill_hashed_kernel(T* __restrict__ dst, int64_t n, uint64_t prefix, float scale) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) Elem<T>::store(dst + i, hashed_value(prefix, (uint64_t)i, scale));
}

template <typename T>
__global__ void fill_const_kernel(T* __restrict__ dst, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) Elem<T>::store(dst + i, v);
}

// Synthetic trunk KV of one layer: element (b, pos, kv head h, dim d), pos < len[b], has index
// (b << 40) + (pos Hkv + h) D + d in tensor `id_k` / `id_v`.  fused != 0: the head-major layouts of the fused pass (keys
// [B][Hkv][stride][64], values transposed per 32-position block), or with pages != null their paged form (block j of
// sequence b in page pages[b * page_stride + j] of a pool [page][Hkv][..]); else [B][stride][Hkv][D].
template <typename T>
__global__ void fill_kv_kernel(T* __restrict__ k, T* __restrict__ v, const int32_t* __restrict__ len, int B, int max_len, int Hkv,
                               int D, int stride, int fused, const int32_t* __restrict__ pages, int page_stride,
                               uint64_t prefix_k, uint64_t prefix_v, float scale) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // over [B][max_len][Hkv][D]
  const int64_t per_seq = (int64_t)max_len * Hkv * D;
  if (i >= per_seq * B) return;
  const int b = (int)(i / per_seq);
  const int64_t r = i - (int64_t)b * per_seq;
  const int pos = (int)(r / (Hkv * D));
  if (pos >= len[b]) return;
  const int h = (int)((r / D) % Hkv), d = (int)(r % D);
  const uint64_t index = ((uint64_t)b << 40) + (uint64_t)r;
  const float kv = hashed_value(prefix_k, index, scale), vv = hashed_value(prefix_v, index, scale);
  if (fused) {
    const int64_t bb = pages ? ((int64_t)pages[b * page_stride + (pos >> 5)] * Hkv + h) * 2048
                             : ((int64_t)b * Hkv + h) * stride * 64 + (int64_t)(pos >> 5) * 2048;
    Elem<T>::store(k + bb + (int64_t)(pos & 31) * 64 + d, kv);
    Elem<T>::store(v + bb + d * 32 + (pos & 31), vv);
  } else {
    const int64_t at = (((int64_t)b * stride + pos) * Hkv + h) * D + d;
    Elem<T>::store(k + at, kv);
    Elem<T>::store(v + at, vv);
  }
}

unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }

}  // namespace

int launch_fill_hashed(int dtype, void* dst, int64_t n, uint64_t seed, uint64_t tensor_id, double std, hipStream_t s) {
  if (n <= 0) return SSD_OK;
  const float scale = (float)(std / kIrwinHallSigma);
  const uint64_t prefix = tensor_prefix(seed, tensor_id);
  if (dtype == SSD_BF16) fill_hashed_kernel<bf16_t><<<blocks_for(n), 256, 0, s>>>((bf16_t*)dst, n, prefix, scale);
  else fill_hashed_kernel<float><<<blocks_for(n), 256, 0, s>>>((float*)dst, n, prefix, scale);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_fill_const(int dtype, void* dst, int64_t n, float v, hipStream_t s) {
  if (n <= 0) return SSD_OK;
  if (dtype == SSD_BF16) fill_const_kernel<bf16_t><<<blocks_for(n), 256, 0, s>>>((bf16_t*)dst, n, v);
  else fill_const_kernel<float><<<blocks_for(n), 256, 0, s>>>((float*)dst, n, v);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_fill_kv(int dtype, void* k, void* v, const int32_t* len, int B, int max_len, int Hkv, int D, int stride, int fused,
                   const int32_t* pages, int page_stride, uint64_t seed, uint64_t id_k, uint64_t id_v, hipStream_t s) {
  const int64_t n = (int64_t)B * max_len * Hkv * D;
  if (n <= 0) return SSD_OK;
  const float scale = (float)(1.0 / kIrwinHallSigma);
  const uint64_t pk = tensor_prefix(seed, id_k), pv = tensor_prefix(seed, id_v);
  if (dtype == SSD_BF16)
    fill_kv_kernel<bf16_t><<<blocks_for(n), 256, 0, s>>>((bf16_t*)k, (bf16_t*)v, len, B, max_len, Hkv, D, stride, fused, pages, page_stride, pk, pv, scale);
  else
    fill_kv_kernel<float><<<blocks_for(n), 256, 0, s>>>((float*)k, (float*)v, len, B, max_len, Hkv, D, stride, fused, pages, page_stride, pk, pv, scale);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

}  // namespace ssd
