// Branch-batched linear layers: y[m][n] = sum_k x[m][k] w[n][k] for a handful of rows m (the branch rows of a
// decode step, or the tokens of an extend) against a large weight matrix that is streamed from HBM once.
//
// bf16 models: MFMA 16x16x32.  The weight matrix is the MFMA A operand (16 output features x 32 inputs per
// instruction), the activations are the B operand (32 inputs x 16 rows).  Weights are kept in HBM in "tile
// order": tile (nt, kt) = 16 features x 32 inputs is 1 KiB, laid out exactly as the 64 lanes hold it (lane l:
// feature nt*16 + l%16, inputs kt*32 + (l/16)*8 .. +7), tiles of one nt consecutive over kt.  A wavefront
// therefore streams its share of a feature tile with fully coalesced 16-byte-per-lane loads.
// Activations arrive as two bf16 planes, head and remainder (x = hi + lo, written by the producing kernel), and
// take two MFMAs per weight tile, so the only bf16 rounding left in a layer is that of the weights themselves
// and of the KV cache.  With a handful of rows the extra MFMAs are free: the kernel is bound by the weight stream.
// fp32 models (the small correctness configuration): plain FMA dot products, one wavefront per output feature.
#include "common.h"

namespace ssd {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kWaves = 4;        // wavefronts per block; they split the reduction dimension
constexpr int kMaxMT = 4;        // 16-row activation tiles per block pass (64 rows)

__global__ void tile_weights_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int N, int Kd) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // one thread per 8-element lane chunk
  int KT = Kd / 32;
  int64_t n_chunks = (int64_t)(N / 16) * KT * 64;
  if (idx >= n_chunks) return;
  int l = (int)(idx & 63);
  int64_t tile = idx >> 6;
  int kt = (int)(tile % KT);
  int64_t nt = tile / KT;
  const bf16_t* s = src + (nt * 16 + (l & 15)) * (int64_t)Kd + kt * 32 + (l >> 4) * 8;
  *(u32x4*)(dst + idx * 8) = *(const u32x4*)s;
}

__device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }

// grid.x = N/16 feature tiles, grid.y = passes of 64 rows.  Each of the 4 wavefronts reduces a quarter of Kd;
// partial tiles meet in LDS; wavefront w finishes activation tile w.
// U = weight tiles a wavefront keeps in flight per stream (gate/up has two streams): 4 KiB did not cover the memory
// latency for the single-stream layers of large models, so they take 8 when the reduction dimension allows.
template <int EPI, int MT, int U>
__global__ __launch_bounds__(kWaves * 64) void gemm_bf16_kernel(const bf16_t* __restrict__ x, int64_t x_plane,
                                                                 const bf16_t* __restrict__ w,
                                                                 const bf16_t* __restrict__ w2, void* __restrict__ out,
                                                                 int64_t ld, int64_t out_plane, int M, int N, int Kd) {
  __shared__ f32x4 red[(EPI == EPI_SWIGLU ? 2 : 1) * kWaves * MT * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nt = blockIdx.x;
  const int m0 = blockIdx.y * (kMaxMT * 16);
  const int KT = Kd / 32;
  const int kt_per_wave = KT / kWaves;
  const int kt0 = wave * kt_per_wave;

  f32x4 acc[MT];
  f32x4 acc2[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) { acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f}; acc2[t] = (f32x4){0.f, 0.f, 0.f, 0.f}; }

  const bf16x8* wp = (const bf16x8*)(w + ((int64_t)nt * KT + kt0) * 512) + lane;
  const bf16x8* wp2 = EPI == EPI_SWIGLU ? (const bf16x8*)(w2 + ((int64_t)nt * KT + kt0) * 512) + lane : nullptr;
  // activation operand: row (clamped to M-1; those columns are never stored), 8 inputs at (lane/16)*8
  const bf16_t* xrow[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    int m = m0 + t * 16 + (lane & 15);
    m = m < M ? m : M - 1;
    xrow[t] = x + (int64_t)m * Kd + (int64_t)kt0 * 32 + (lane >> 4) * 8;
  }

  // Two register sets of U tiles per stream: the next group's weight loads go out before the current group is
  // multiplied, so a wavefront always has a group in flight (with one set the wavefront idled for a memory round trip per
  // group, and the layers with few feature tiles per compute unit had nobody else to fill it).
  auto load_group = [&](bf16x8* wr, bf16x8* wr2, int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      wr[u] = __builtin_nontemporal_load(wp + (int64_t)(kt + u) * 64);
      if (EPI == EPI_SWIGLU) wr2[u] = __builtin_nontemporal_load(wp2 + (int64_t)(kt + u) * 64);
    }
  };
  auto mfma_group = [&](const bf16x8* wr, const bf16x8* wr2, int kt) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        bf16x8 hi = *(const bf16x8*)(xrow[t] + (kt + u) * 32);
        bf16x8 lo = *(const bf16x8*)(xrow[t] + x_plane + (kt + u) * 32);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wr[u], hi, acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wr[u], lo, acc[t], 0, 0, 0);
        if (EPI == EPI_SWIGLU) {
          acc2[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wr2[u], hi, acc2[t], 0, 0, 0);
          acc2[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wr2[u], lo, acc2[t], 0, 0, 0);
        }
      }
    }
  };
  bf16x8 wa[U], wa2[U], wb[U], wb2[U];
  const int n_groups = kt_per_wave / U;            // kt_per_wave is a multiple of U (host check)
  if (n_groups > 0) load_group(wa, wa2, 0);
  int g = 0;
  for (; g + 2 <= n_groups; g += 2) {
    load_group(wb, wb2, (g + 1) * U);
    mfma_group(wa, wa2, g * U);
    if (g + 2 < n_groups) load_group(wa, wa2, (g + 2) * U);
    mfma_group(wb, wb2, (g + 1) * U);
  }
  if (g < n_groups) mfma_group(wa, wa2, g * U);    // odd number of groups: the last one is already in wa

#pragma unroll
  for (int t = 0; t < MT; ++t) {
    red[(wave * MT + t) * 64 + lane] = acc[t];
    if (EPI == EPI_SWIGLU) red[kWaves * MT * 64 + (wave * MT + t) * 64 + lane] = acc2[t];
  }
  __syncthreads();
  for (int t = wave; t < MT; t += kWaves) {
    f32x4 sum = red[t * 64 + lane];
#pragma unroll
    for (int v = 1; v < kWaves; ++v) sum += red[(v * MT + t) * 64 + lane];
    int m = m0 + t * 16 + (lane & 15);
    int n = nt * 16 + (lane >> 4) * 4;
    if (m >= M) continue;
    if (EPI == EPI_STORE_F32) {
      *(f32x4*)((float*)out + (int64_t)m * ld + n) = sum;
    } else if (EPI == EPI_RESIDUAL_ADD) {
      f32x4* p = (f32x4*)((float*)out + (int64_t)m * ld + n);
      *p = *p + sum;
    } else {
      f32x4 up = red[kWaves * MT * 64 + t * 64 + lane];
#pragma unroll
      for (int v = 1; v < kWaves; ++v) up += red[kWaves * MT * 64 + (v * MT + t) * 64 + lane];
#pragma unroll
      for (int r = 0; r < 4; ++r) Act<bf16_t>::store(out, out_plane, (int64_t)m * ld + n + r, silu(sum[r]) * up[r]);
    }
  }
}

// fp32: one wavefront per output feature, lanes stride over the inputs, up to 16 rows per pass.
constexpr int kRowsF32 = 16;
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                        const float* __restrict__ w2, float* __restrict__ out, int64_t ld,
                                                        int M, int N, int Kd) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 4 + wave;
  const int m0 = blockIdx.y * kRowsF32;
  if (n >= N) return;
  float acc[kRowsF32], acc2[kRowsF32];
#pragma unroll
  for (int r = 0; r < kRowsF32; ++r) { acc[r] = 0.f; acc2[r] = 0.f; }
  const float* wrow = w + (int64_t)n * Kd;
  const float* wrow2 = EPI == EPI_SWIGLU ? w2 + (int64_t)n * Kd : nullptr;
  for (int k = lane; k < Kd; k += 64) {
    float wv = wrow[k];
    float wv2 = EPI == EPI_SWIGLU ? wrow2[k] : 0.f;
#pragma unroll
    for (int r = 0; r < kRowsF32; ++r) {
      int m = m0 + r;
      float xv = m < M ? x[(int64_t)m * Kd + k] : 0.f;
      acc[r] = fmaf(xv, wv, acc[r]);
      if (EPI == EPI_SWIGLU) acc2[r] = fmaf(xv, wv2, acc2[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < kRowsF32; ++r) {
    float v = acc[r], v2 = acc2[r];
    for (int o = 32; o > 0; o >>= 1) {
      v += __shfl_xor(v, o);
      if (EPI == EPI_SWIGLU) v2 += __shfl_xor(v2, o);
    }
    int m = m0 + r;
    if (lane == 0 && m < M) {
      float* p = out + (int64_t)m * ld + n;
      if (EPI == EPI_STORE_F32) *p = v;
      else if (EPI == EPI_RESIDUAL_ADD) *p += v;
      else *p = (v / (1.0f + expf(-v))) * v2;
    }
  }
}

template <int EPI>
int launch_bf16(const void* x, int64_t x_plane, const void* w, const void* w2, void* out, int64_t ld, int64_t out_plane,
                int M, int N, int Kd, hipStream_t s) {
  dim3 grid(N / 16, (M + kMaxMT * 16 - 1) / (kMaxMT * 16));
  int rows_in_pass = M < kMaxMT * 16 ? M : kMaxMT * 16;
  int mt = (rows_in_pass + 15) / 16;
  const bf16_t *xb = (const bf16_t*)x, *wb = (const bf16_t*)w, *w2b = (const bf16_t*)w2;
  const bool deep = EPI != EPI_SWIGLU && (Kd / 32 / kWaves) % 8 == 0;
#define SSD_GEMM_LAUNCH(MTV)                                                                                             \
  do {                                                                                                                   \
    if (deep) gemm_bf16_kernel<EPI, MTV, 8><<<grid, kWaves * 64, 0, s>>>(xb, x_plane, wb, w2b, out, ld, out_plane, M, N, Kd); \
    else gemm_bf16_kernel<EPI, MTV, 4><<<grid, kWaves * 64, 0, s>>>(xb, x_plane, wb, w2b, out, ld, out_plane, M, N, Kd);      \
  } while (0)
  switch (mt) {
    case 1: SSD_GEMM_LAUNCH(1); break;
    case 2: SSD_GEMM_LAUNCH(2); break;
    case 3: SSD_GEMM_LAUNCH(3); break;
    default: SSD_GEMM_LAUNCH(4); break;
  }
#undef SSD_GEMM_LAUNCH
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

template <int EPI>
int launch_f32(const void* x, const void* w, const void* w2, void* out, int64_t ld, int M, int N, int Kd, hipStream_t s) {
  dim3 grid((N + 3) / 4, (M + kRowsF32 - 1) / kRowsF32);
  gemm_f32_kernel<EPI><<<grid, 256, 0, s>>>((const float*)x, (const float*)w, (const float*)w2, (float*)out, ld, M, N, Kd);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

}  // namespace

int launch_tile_weights_bf16(const bf16_t* src, bf16_t* dst, int N, int Kd, hipStream_t s) {
  SSD_CHECK_ARG(N % 16 == 0 && Kd % (32 * kWaves * 4) == 0,
                "bf16 weight %d x %d: features must be a multiple of 16 and inputs of %d", N, Kd, 32 * kWaves * 4);
  int64_t n_chunks = (int64_t)(N / 16) * (Kd / 32) * 64;
  tile_weights_kernel<<<(int)((n_chunks + 255) / 256), 256, 0, s>>>(src, dst, N, Kd);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_gemm(int dtype, int epi, const void* x, int64_t x_plane, const void* w, const void* w2, void* out, int64_t ld,
                int64_t out_plane, int M, int N, int Kd, hipStream_t s) {
  if (M <= 0) return SSD_OK;
  if (dtype == SSD_BF16) {
    switch (epi) {
      case EPI_STORE_F32: return launch_bf16<EPI_STORE_F32>(x, x_plane, w, w2, out, ld, out_plane, M, N, Kd, s);
      case EPI_RESIDUAL_ADD: return launch_bf16<EPI_RESIDUAL_ADD>(x, x_plane, w, w2, out, ld, out_plane, M, N, Kd, s);
      default: return launch_bf16<EPI_SWIGLU>(x, x_plane, w, w2, out, ld, out_plane, M, N, Kd, s);
    }
  }
  switch (epi) {
    case EPI_STORE_F32: return launch_f32<EPI_STORE_F32>(x, w, w2, out, ld, M, N, Kd, s);
    case EPI_RESIDUAL_ADD: return launch_f32<EPI_RESIDUAL_ADD>(x, w, w2, out, ld, M, N, Kd, s);
    default: return launch_f32<EPI_SWIGLU>(x, w, w2, out, ld, M, N, Kd, s);
  }
}

}  // namespace ssd
