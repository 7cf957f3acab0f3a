// Selection kernels: top-F bonus-token candidates per accept length (Sec. 4.1.1), the branch sampler
// (argmax / Gumbel-max), and lossless verification (Sec. 2.1).  All orderings are (score descending,
// token id ascending); NaN ranks below every number.
#include <mutex>

#include "common.h"
#include "rng.h"

namespace ssd {

namespace {

constexpr int kSelBlock = 1024;
constexpr int kSelWaves = kSelBlock / 64;

// 64-bit sort key of (fp32 logit, token id): larger key = better candidate.
__device__ __forceinline__ uint64_t make_key(float f, int id) {
  uint32_t hi;
  if (f != f) hi = 0u;                              // NaN: below -inf
  else {
    if (f == 0.f) f = 0.f;                          // -0 and +0 tie
    uint32_t u = __float_as_uint(f);
    hi = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  }
  return ((uint64_t)hi << 32) | (uint32_t)(~(uint32_t)id);
}
__device__ __forceinline__ int key_id(uint64_t k) { return (int)(~(uint32_t)k); }

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
  for (int o = 32; o > 0; o >>= 1) {
    uint64_t t = __shfl_xor((unsigned long long)v, o);
    v = t > v ? t : v;
  }
  return v;
}

// One block per row.  Every thread keeps the best FMAX keys of its strided share in sorted registers; then F
// rounds of a block-wide maximum over the threads' current heads pick the row's top F in order.
// groups == 0: every row takes F ids, stored at ids[row][F].  groups == K+1 (the fan-out of a round, Sec. 4.1.1 with
// the cache shape of Sec. 4.1.2): row (b, k) takes F_k ids, stored at ids[b][off[k] ..].
// gridDim.y > 1: the vocabulary is cut into gridDim.y parts, block (row, part) leaves the sorted keys of its part's
// top F in part_keys[row][part][FMAX] and top_f_merge_kernel picks the row's top F among them (keys are unique, so
// the result is the same as that of one block).
constexpr int kTopFMaxParts = 32;
template <int FMAX>
__global__ __launch_bounds__(kSelBlock) void top_f_kernel(const float* __restrict__ logits, int64_t ld,
                                                          const int32_t* __restrict__ exclude, int V, int F, int groups,
                                                          FanTable fan, int32_t* __restrict__ ids,
                                                          uint64_t* __restrict__ part_keys) {
  __shared__ uint64_t wave_best[kSelWaves];
  __shared__ uint64_t round_best;
  const int row = blockIdx.x;
  const int parts = gridDim.y, part = blockIdx.y;
  int32_t* out = ids + (int64_t)row * F;
  if (groups > 0) {
    const int b = row / groups, k = row - b * groups;
    F = fan.off[k + 1] - fan.off[k];
    out = ids + (int64_t)b * fan.off[groups] + fan.off[k];
  }
  const int chunk = (V + parts - 1) / parts;
  const int lo = part * chunk, hi = lo + chunk < V ? lo + chunk : V;
  const float* z = logits + (int64_t)row * ld;
  const int ex = exclude ? exclude[row] : -1;
  uint64_t best[FMAX];
#pragma unroll
  for (int i = 0; i < FMAX; ++i) best[i] = 0ull;    // 0 is below every real key (ids < 2^32-1)
  auto offer = [&](float v, int t) {
    if (t == ex) return;
    uint64_t k = make_key(v, t);
    if (k > best[FMAX - 1]) {
      best[FMAX - 1] = k;
#pragma unroll
      for (int i = FMAX - 1; i > 0; --i) {
        if (best[i] > best[i - 1]) { uint64_t tmp = best[i]; best[i] = best[i - 1]; best[i - 1] = tmp; }
      }
    }
  };
  // eight loads in flight per thread: one dependent load per iteration would cost a memory latency each
  constexpr int U = 8;
  for (int t0 = lo + threadIdx.x; t0 < hi; t0 += kSelBlock * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * kSelBlock;
      v[u] = z[t < hi ? t : t0];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * kSelBlock;
      if (t < hi) offer(v[u], t);
    }
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int f = 0; f < F; ++f) {
    uint64_t w = wave_max_u64(best[0]);
    if (lane == 0) wave_best[wave] = w;
    __syncthreads();
    if (wave == 0) {
      uint64_t v = lane < kSelWaves ? wave_best[lane] : 0ull;
      v = wave_max_u64(v);
      if (lane == 0) {
        round_best = v;
        if (parts == 1) out[f] = key_id(v);
        else part_keys[((int64_t)row * parts + part) * FMAX + f] = v;     // 0 when the part ran out of tokens
      }
    }
    __syncthreads();
    if (best[0] == round_best) {                    // keys are unique: exactly one thread pops
#pragma unroll
      for (int i = 0; i < FMAX - 1; ++i) best[i] = best[i + 1];
      best[FMAX - 1] = 0ull;
    }
  }
}

// One wavefront per row: the top F of the parts' candidates.  Keys are unique and positive, 0 marks "none".
template <int FMAX>
__global__ __launch_bounds__(64) void top_f_merge_kernel(const uint64_t* __restrict__ part_keys, int parts, int F, int groups,
                                                          FanTable fan, int32_t* __restrict__ ids) {
  const int row = blockIdx.x, lane = threadIdx.x;
  int32_t* out = ids + (int64_t)row * F;
  if (groups > 0) {
    const int b = row / groups, k = row - b * groups;
    F = fan.off[k + 1] - fan.off[k];
    out = ids + (int64_t)b * fan.off[groups] + fan.off[k];
  }
  constexpr int PER = kTopFMaxParts * FMAX / 64;      // candidates per lane
  uint64_t mine[PER];
  const int n = parts * F;                            // part p holds its F best at [p][0..F-1]
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int c = lane + 64 * i;
    mine[i] = c < n ? part_keys[((int64_t)row * parts + c / F) * FMAX + c % F] : 0ull;
  }
  uint64_t prev = ~0ull;
  for (int f = 0; f < F; ++f) {
    uint64_t best = 0ull;
#pragma unroll
    for (int i = 0; i < PER; ++i) best = mine[i] < prev && mine[i] > best ? mine[i] : best;
    best = wave_max_u64(best);
    if (lane == 0) out[f] = key_id(best);
    prev = best;
  }
}

struct ScoreId {
  double s;
  int id;
};
constexpr int kSampleMaxParts = 64;   // blocks that share one row of the sampler
__device__ __forceinline__ bool better(const ScoreId& a, const ScoreId& b) {
  return a.s > b.s || (a.s == b.s && a.id < b.id);
}
__device__ __forceinline__ ScoreId block_argmax(ScoreId v, ScoreId* smem) {
  for (int o = 32; o > 0; o >>= 1) {
    ScoreId t;
    t.s = __shfl_xor(v.s, o);
    t.id = __shfl_xor(v.id, o);
    if (better(t, v)) v = t;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) smem[wave] = v;
  __syncthreads();
  ScoreId r = smem[0];
  for (int i = 1; i < kSelWaves; ++i)
    if (better(smem[i], r)) r = smem[i];
  __syncthreads();
  return r;
}
__device__ __forceinline__ double block_sum_f64(double v, double* smem) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) smem[wave] = v;
  __syncthreads();
  double r = 0.0;
  for (int i = 0; i < kSelWaves; ++i) r += smem[i];
  __syncthreads();
  return r;
}
__device__ __forceinline__ double score_of(float z) { return z != z ? -INFINITY : (double)z; }

// Branch sampler: greedy argmax or Gumbel-max sample of softmax(z / T).  grid = (rows, parts): a block scans one
// part of its row's vocabulary; with one part it writes the token, otherwise its best (score, id) goes to `scratch`
// [row][part] and sample_merge_kernel picks the row's winner (the order `better` defines is total, so any grouping
// gives the same token).
__global__ __launch_bounds__(kSelBlock) void sample_kernel(const float* __restrict__ logits, int64_t ld,
                                                           const float* __restrict__ temperature, int rows_per_seq,
                                                           int V, uint64_t seed, int row_base, int step,
                                                           int32_t* __restrict__ out, int64_t out_stride,
                                                           ScoreId* __restrict__ scratch, int exact_scan) {
  __shared__ ScoreId smem[kSelWaves];
  const int row = blockIdx.x, part = blockIdx.y, parts = gridDim.y;
  const float* z = logits + (int64_t)row * ld;
  const double T = (double)temperature[row / rows_per_seq];
  const uint64_t prefix = draw_prefix(seed, STREAM_DRAFT, (uint64_t)(row_base + row), (uint64_t)step);
  // this block's share of the vocabulary, in groups of 4 tokens
  const int n4_all = (V + 3) >> 2;
  const int per = (n4_all + parts - 1) / parts;
  const int q_begin = part * per, q_end = min(n4_all, q_begin + per);
  ScoreId best = {-INFINITY, 0x7fffffff};
  if (T <= 0.0 && (V & 3) == 0 && (ld & 3) == 0 && ((uintptr_t)logits & 15) == 0) {
    // greedy rows: 16-byte loads, eight of them in flight per thread (one dependent 4-byte load per iteration
    // would cost a memory latency each)
    typedef __attribute__((ext_vector_type(4))) float f4;
    const f4* z4 = (const f4*)z;
    for (int t0 = q_begin + threadIdx.x; t0 < q_end; t0 += kSelBlock * 8) {
      f4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int t = t0 + u * kSelBlock;
        v[u] = z4[t < q_end ? t : t0];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int t = t0 + u * kSelBlock;
        if (t < q_end) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            ScoreId c = {score_of(v[u][e]), t * 4 + e};
            if (better(c, best)) best = c;
          }
        }
      }
    }
  } else if (T <= 0.0 || exact_scan) {
    const int t_end = min(V, q_end * 4);
    for (int t = q_begin * 4 + threadIdx.x; t < t_end; t += kSelBlock) {
      ScoreId c;
      c.id = t;
      c.s = score_of(z[t]);
      if (T > 0.0) c.s = c.s / T + gumbel_from_u(draw_u(prefix, (uint64_t)t));
      if (better(c, best)) best = c;
    }
  } else {
    // Sampled rows.  The decision is the fp64 one (score = z / T + g in double, as specified), but two fp64 logarithms
    // per token of a 128256-token row cost more than the rest of the sampler together, so the scan runs in fp32 and
    // only the tokens that can still win are scored in fp64: with |s32 - s64| <= delta for every token near the top,
    // the fp64 winner t* has s32(t*) >= s64(t*) - delta >= s64(t32) - delta >= max32 - 2 delta.  delta: z / T in
    // fp32 is within 2^-22 |z / T|; u is exact in fp32 (a 24-bit odd integer times 2^-24); logf is good to 2 ulp, so
    // g = -log(-log u) (at most 16.7 in magnitude) to 5e-6; near the top |z / T| <= |s| + 17.  The bound used is
    // twice that.
    const int t_begin = q_begin * 4, t_end = min(V, q_end * 4);
    const float inv_t = 1.0f / (float)T;
    auto s32 = [&](int t) {
      const float zt = z[t];
      if (zt != zt) return -INFINITY;
      const uint64_t m = mix64(prefix + (uint64_t)t) >> 41;
      const float u = ((float)m + 0.5f) * (1.0f / 8388608.0f);
      return zt * inv_t - logf(-logf(u));
    };
    float mx = -INFINITY;
    for (int t = t_begin + threadIdx.x; t < t_end; t += kSelBlock) mx = fmaxf(mx, s32(t));
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    __shared__ float fmx[kSelWaves];
    if ((threadIdx.x & 63) == 0) fmx[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmx[0];
    for (int i = 1; i < kSelWaves; ++i) mx = fmaxf(mx, fmx[i]);
    // an infinite or empty maximum: score everything in fp64
    const float thr = mx > -INFINITY && mx < INFINITY ? mx - 2.0f * (2e-6f * (fabsf(mx) + 40.0f) + 2e-5f) : -INFINITY;
    for (int t = t_begin + threadIdx.x; t < t_end; t += kSelBlock) {
      if (s32(t) >= thr) {
        ScoreId c;
        c.id = t;
        c.s = score_of(z[t]) / T + gumbel_from_u(draw_u(prefix, (uint64_t)t));
        if (better(c, best)) best = c;
      }
    }
  }
  best = block_argmax(best, smem);
  if (threadIdx.x == 0) {
    if (parts == 1) out[(int64_t)row * out_stride] = best.id;
    else scratch[(int64_t)row * parts + part] = best;
  }
}

__global__ __launch_bounds__(64) void sample_merge_kernel(const ScoreId* __restrict__ scratch, int parts,
                                                          int32_t* __restrict__ out, int64_t out_stride) {
  const int row = blockIdx.x;
  ScoreId best = {-INFINITY, 0x7fffffff};
  for (int i = threadIdx.x; i < parts; i += 64) {
    const ScoreId c = scratch[(int64_t)row * parts + i];
    if (better(c, best)) best = c;
  }
  for (int o = 32; o > 0; o >>= 1) {
    ScoreId t;
    t.s = __shfl_xor(best.s, o);
    t.id = __shfl_xor(best.id, o);
    if (better(t, best)) best = t;
  }
  if (threadIdx.x == 0) out[(int64_t)row * out_stride] = best.id;
}

struct RowStats {
  double max;     // max of the row's logits
  double sum;     // sum exp((z - max)/T), T > 0 only
  int32_t argmax;
  int32_t pad;
};

// ---- lossless verification (Sec. 2.1).  Every pass over a row of logits is shared among `parts` blocks, so that
// the few rows of one verification occupy the whole chip; partial results meet in the workspace and are merged in a
// fixed order (the result does not depend on timing).
constexpr int kVerifyMaxParts = 32;
struct VerifyWs {
  RowStats* stats;        // [B (2K+1)]: target rows 0..K, then draft rows 0..K-1 of each sequence
  ScoreId* part_best;     // [rows][parts]
  double* part_sum;       // [rows][parts]
  double* part_mass;      // [B][parts]  residual mass of the bonus position
  ScoreId* part_bonus;    // [B][parts]
  int32_t* accept;        // [B]
};
__host__ __device__ inline size_t verify_ws_align(size_t x) { return (x + 15) & ~(size_t)15; }
__host__ inline VerifyWs verify_ws_carve(void* base, int B, int K) {
  const size_t rows = (size_t)B * (2 * K + 1);
  char* p = (char*)base;
  VerifyWs w;
  w.stats = (RowStats*)p;      p += verify_ws_align(rows * sizeof(RowStats));
  w.part_best = (ScoreId*)p;   p += verify_ws_align(rows * kVerifyMaxParts * sizeof(ScoreId));
  w.part_sum = (double*)p;     p += verify_ws_align(rows * kVerifyMaxParts * sizeof(double));
  w.part_mass = (double*)p;    p += verify_ws_align((size_t)B * kVerifyMaxParts * sizeof(double));
  w.part_bonus = (ScoreId*)p;  p += verify_ws_align((size_t)B * kVerifyMaxParts * sizeof(ScoreId));
  w.accept = (int32_t*)p;
  return w;
}

// the logit row of workspace row r of sequence b (nullptr: a draft row of a greedy sequence, nothing to do)
__device__ __forceinline__ const float* verify_row(const float* zt, const float* zd, int b, int r, int K, int V, double T) {
  if (r <= K) return zt + ((int64_t)b * (K + 1) + r) * V;
  if (T <= 0.0) return nullptr;
  return zd + ((int64_t)b * K + (r - K - 1)) * V;
}
// this block's share [lo, hi) of a vocabulary of V tokens
__device__ __forceinline__ void verify_share(int V, int& lo, int& hi) {
  const int chunk = (V + (int)gridDim.y - 1) / (int)gridDim.y;
  lo = (int)blockIdx.y * chunk;
  hi = lo + chunk < V ? lo + chunk : V;
}

// Pass 1: per logit row and part, the best (logit, token).  grid (B (2K+1), parts).
__global__ __launch_bounds__(kSelBlock) void verify_max_kernel(const float* __restrict__ zt, const float* __restrict__ zd,
                                                               const float* __restrict__ temperature, int K, int V,
                                                               VerifyWs ws) {
  __shared__ ScoreId smem[kSelWaves];
  const int b = blockIdx.x / (2 * K + 1), r = blockIdx.x % (2 * K + 1);
  const double T = zd ? (double)temperature[b] : 0.0;   // without draft logits every sequence is greedy
  const float* z = verify_row(zt, zd, b, r, K, V, T);
  if (!z) return;
  int lo, hi;
  verify_share(V, lo, hi);
  ScoreId best = {-INFINITY, 0x7fffffff};
  constexpr int U = 8;   // loads in flight per thread
  for (int t0 = lo + threadIdx.x; t0 < hi; t0 += kSelBlock * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * kSelBlock;
      v[u] = z[t < hi ? t : t0];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * kSelBlock;
      ScoreId c = {score_of(v[u]), t};
      if (t < hi && better(c, best)) best = c;
    }
  }
  best = block_argmax(best, smem);
  if (threadIdx.x == 0) ws.part_best[(int64_t)blockIdx.x * gridDim.y + blockIdx.y] = best;
}

// the row's best over the parts of pass 1 (every thread of the block computes the same)
__device__ __forceinline__ ScoreId verify_row_best(const VerifyWs& ws, int64_t row, int parts) {
  ScoreId best = ws.part_best[row * parts];
  for (int i = 1; i < parts; ++i) {
    const ScoreId c = ws.part_best[row * parts + i];
    if (better(c, best)) best = c;
  }
  return best;
}

// Pass 2: per row and part, the partial softmax denominator sum exp((z - max) / T); part 0 also records the row's
// max and argmax.  grid (B (2K+1), parts).
__global__ __launch_bounds__(kSelBlock) void verify_sum_kernel(const float* __restrict__ zt, const float* __restrict__ zd,
                                                               const float* __restrict__ temperature, int K, int V,
                                                               VerifyWs ws) {
  __shared__ double dsm[kSelWaves];
  const int b = blockIdx.x / (2 * K + 1), r = blockIdx.x % (2 * K + 1);
  const double T = zd ? (double)temperature[b] : 0.0;
  const float* z = verify_row(zt, zd, b, r, K, V, T);
  if (!z) return;
  const ScoreId best = verify_row_best(ws, blockIdx.x, gridDim.y);
  if (blockIdx.y == 0 && threadIdx.x == 0) {
    ws.stats[blockIdx.x].max = best.s;
    ws.stats[blockIdx.x].argmax = best.id;
    ws.stats[blockIdx.x].pad = 0;
  }
  if (T <= 0.0) return;
  int lo, hi;
  verify_share(V, lo, hi);
  double sum = 0.0;
  constexpr int U = 8;
  for (int t0 = lo + threadIdx.x; t0 < hi; t0 += kSelBlock * U) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * kSelBlock;
      v[u] = z[t < hi ? t : t0];
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (t0 + u * kSelBlock < hi) sum += exp((score_of(v[u]) - best.s) / T);
  }
  sum = block_sum_f64(sum, dsm);
  if (threadIdx.x == 0) ws.part_sum[(int64_t)blockIdx.x * gridDim.y + blockIdx.y] = sum;
}

// Pass 3: the sequential acceptance (one thread per sequence of work, done by every block of the sequence so that
// all of them know the bonus position k), then this part's share of the residual mass at position k.  Part 0
// publishes k, and the bonus token itself if the sequence is greedy.  grid (B, parts).
__global__ __launch_bounds__(kSelBlock) void verify_accept_kernel(const float* __restrict__ zt, const float* __restrict__ zd,
                                                                  const int32_t* __restrict__ spec,
                                                                  const float* __restrict__ temperature, int K, int V,
                                                                  uint64_t seed, VerifyWs ws, int row_parts,
                                                                  int32_t* __restrict__ accept_len,
                                                                  int32_t* __restrict__ bonus) {
  __shared__ double dsm[kSelWaves];
  __shared__ int k_s;
  const int b = blockIdx.x, parts = gridDim.y;   // row_parts: the parts passes 1 and 2 cut a row into (may differ)
  const double T = zd ? (double)temperature[b] : 0.0;
  RowStats* st = ws.stats + (int64_t)b * (2 * K + 1);
  // the rows' softmax denominators: the parts' sums in part order (threads 0 .. 2K merge one row each; part 0 keeps them)
  __shared__ double sums[2 * SSD_MAX_K + 1];
  if (T > 0.0 && (int)threadIdx.x <= 2 * K) {
    const int64_t row = (int64_t)b * (2 * K + 1) + threadIdx.x;
    double sum = 0.0;
    for (int i = 0; i < row_parts; ++i) sum += ws.part_sum[row * row_parts + i];
    sums[threadIdx.x] = sum;
    if (blockIdx.y == 0) st[threadIdx.x].sum = sum;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int k = K;
    for (int i = 0; i < K; ++i) {
      int s = spec[(int64_t)b * K + i];
      bool ok;
      if (T <= 0.0) ok = st[i].argmax == s;
      else if (s < 0 || s >= V) ok = false;
      else {
        double p = exp((score_of(zt[((int64_t)b * (K + 1) + i) * V + s]) - st[i].max) / T) / sums[i];
        double q = exp((score_of(zd[((int64_t)b * K + i) * V + s]) - st[K + 1 + i].max) / T) / sums[K + 1 + i];
        double u = draw_u(draw_prefix(seed, STREAM_ACCEPT, (uint64_t)b, (uint64_t)i), 0ull);
        ok = u * q < p;
      }
      if (!ok) { k = i; break; }
    }
    k_s = k;
  }
  __syncthreads();
  const int k = k_s;
  if (blockIdx.y == 0 && threadIdx.x == 0) {
    ws.accept[b] = k;
    accept_len[b] = k;
    if (T <= 0.0) bonus[b] = st[k].argmax;
  }
  if (T <= 0.0) return;
  double mass = 0.0;
  if (k < K) {
    const float* zp = zt + ((int64_t)b * (K + 1) + k) * V;
    const float* zq = zd + ((int64_t)b * K + k) * V;
    const double pmax = st[k].max, psum = sums[k], qmax = st[K + 1 + k].max, qsum = sums[K + 1 + k];
    int lo, hi;
    verify_share(V, lo, hi);
    for (int t = lo + threadIdx.x; t < hi; t += kSelBlock) {
      double p = exp((score_of(zp[t]) - pmax) / T) / psum;
      double q = exp((score_of(zq[t]) - qmax) / T) / qsum;
      mass += fmax(p - q, 0.0);
    }
    mass = block_sum_f64(mass, dsm);
  }
  if (threadIdx.x == 0) ws.part_mass[(int64_t)b * parts + blockIdx.y] = mass;
}

// Pass 4: this part's best Gumbel-max candidate for the bonus token at position k: from the residual max(p - q, 0)
// if it has mass (k < K), else from p.  grid (B, parts); greedy sequences are done already.
__global__ __launch_bounds__(kSelBlock) void verify_bonus_kernel(const float* __restrict__ zt, const float* __restrict__ zd,
                                                                 const float* __restrict__ temperature, int K, int V,
                                                                 uint64_t seed, VerifyWs ws) {
  __shared__ ScoreId smem[kSelWaves];
  const int b = blockIdx.x, parts = gridDim.y;
  const double T = zd ? (double)temperature[b] : 0.0;
  if (T <= 0.0) return;
  const RowStats* st = ws.stats + (int64_t)b * (2 * K + 1);
  const int k = ws.accept[b];
  double total = 0.0;
  for (int i = 0; i < parts; ++i) total += ws.part_mass[(int64_t)b * parts + i];
  const bool use_residual = k < K && total > 0.0;
  const float* zp = zt + ((int64_t)b * (K + 1) + k) * V;
  const float* zq = k < K ? zd + ((int64_t)b * K + k) * V : nullptr;
  const double pmax = st[k].max, psum = st[k].sum;
  const double qmax = k < K ? st[K + 1 + k].max : 0.0, qsum = k < K ? st[K + 1 + k].sum : 1.0;
  const uint64_t prefix = draw_prefix(seed, STREAM_BONUS, (uint64_t)b, (uint64_t)k);
  int lo, hi;
  verify_share(V, lo, hi);
  ScoreId best = {-INFINITY, 0x7fffffff};
  for (int t = lo + threadIdx.x; t < hi; t += kSelBlock) {
    double r = exp((score_of(zp[t]) - pmax) / T) / psum;
    if (use_residual) r = fmax(r - exp((score_of(zq[t]) - qmax) / T) / qsum, 0.0);
    ScoreId c;
    c.id = t;
    c.s = r > 0.0 ? log(r) + gumbel_from_u(draw_u(prefix, (uint64_t)t)) : -INFINITY;
    if (better(c, best)) best = c;
  }
  best = block_argmax(best, smem);
  if (threadIdx.x == 0) ws.part_bonus[(int64_t)b * parts + blockIdx.y] = best;
}

// Pass 5: the bonus token of every sampled sequence among its parts' candidates.  One wavefront per sequence.
__global__ __launch_bounds__(64) void verify_bonus_merge_kernel(const float* __restrict__ zd, const float* __restrict__ temperature,
                                                                int parts, VerifyWs ws, int32_t* __restrict__ bonus) {
  const int b = blockIdx.x;
  if (!(zd && temperature[b] > 0.f)) return;
  ScoreId best = {-INFINITY, 0x7fffffff};
  for (int i = threadIdx.x; i < parts; i += 64) {
    const ScoreId c = ws.part_bonus[(int64_t)b * parts + i];
    if (better(c, best)) best = c;
  }
  for (int o = 32; o > 0; o >>= 1) {
    ScoreId t;
    t.s = __shfl_xor(best.s, o);
    t.id = __shfl_xor(best.id, o);
    if (better(t, best)) best = t;
  }
  if (threadIdx.x == 0) bonus[b] = best.id;
}

}  // namespace

namespace {

// Parts per row: enough blocks to occupy the chip when there are few rows, at least 4096 tokens per part.
int top_f_parts(int rows, int V, const void* scratch) {
  if (!scratch) return 1;
  int parts = 512 / rows;
  parts = parts > kTopFMaxParts ? kTopFMaxParts : parts;
  while (parts > 1 && V / parts < 4096) --parts;
  return parts < 1 ? 1 : parts;
}

template <int FMAX>
int run_top_f(const float* logits, int64_t ld, const int32_t* exclude, int rows, int V, int F, int groups, const FanTable& fan,
              int32_t* ids, void* scratch, hipStream_t s) {
  const int parts = top_f_parts(rows, V, scratch);
  top_f_kernel<FMAX><<<dim3(rows, parts), kSelBlock, 0, s>>>(logits, ld, exclude, V, F, groups, fan, ids, (uint64_t*)scratch);
  if (parts > 1) top_f_merge_kernel<FMAX><<<rows, 64, 0, s>>>((const uint64_t*)scratch, parts, F, groups, fan, ids);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

}  // namespace

size_t top_f_scratch_bytes(int rows) { return (size_t)rows * kTopFMaxParts * SSD_MAX_F * sizeof(uint64_t); }

int launch_top_f(const float* logits, int64_t ld, const int32_t* exclude, int rows, int V, int F, int32_t* ids,
                 void* scratch, hipStream_t s) {
  if (rows <= 0) return SSD_OK;
  const FanTable none = {};
  if (F <= 4) return run_top_f<4>(logits, ld, exclude, rows, V, F, 0, none, ids, scratch, s);
  if (F <= 8) return run_top_f<8>(logits, ld, exclude, rows, V, F, 0, none, ids, scratch, s);
  return run_top_f<16>(logits, ld, exclude, rows, V, F, 0, none, ids, scratch, s);
}

// Random-token backup speculator (Sec. 4.3): token i of sequence b is the 64-bit hash of (seed, backup stream, b, i, 0)
// modulo the vocabulary size.
__global__ void backup_random_kernel(int32_t* __restrict__ tokens, int B, int K, int V, uint64_t seed) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= B * K) return;
  const int b = idx / K, i = idx - b * K;
  tokens[idx] = (int32_t)(mix64(draw_prefix(seed, STREAM_BACKUP, (uint64_t)b, (uint64_t)i)) % (uint64_t)V);
}

int launch_backup_random(int32_t* tokens, int B, int K, int V, uint64_t seed, hipStream_t s) {
  if (B * K <= 0) return SSD_OK;
  backup_random_kernel<<<(B * K + 255) / 256, 256, 0, s>>>(tokens, B, K, V, seed);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_top_f_fan(const float* logits, int64_t ld, const int32_t* exclude, int B, int K, const FanTable& fan, int V,
                     int32_t* ids, void* scratch, hipStream_t s) {
  const int rows = B * (K + 1);
  if (rows <= 0) return SSD_OK;
  int f_max = 0;
  for (int k = 0; k <= K; ++k) f_max = fan.off[k + 1] - fan.off[k] > f_max ? fan.off[k + 1] - fan.off[k] : f_max;
  if (f_max <= 4) return run_top_f<4>(logits, ld, exclude, rows, V, 0, K + 1, fan, ids, scratch, s);
  if (f_max <= 8) return run_top_f<8>(logits, ld, exclude, rows, V, 0, K + 1, fan, ids, scratch, s);
  return run_top_f<16>(logits, ld, exclude, rows, V, 0, K + 1, fan, ids, scratch, s);
}

// Saguaro sampling scheme sigma_{F,C} (Sec. 4.2.1) on rows of logits, in place: the F tokens in ids[row] (the row's own
// top-F) get T log C added, which multiplies their weight exp(z/T) by C.  Greedy rows (T == 0) are left alone.
__global__ void sigma_shift_kernel(float* __restrict__ logits, int64_t ld, const float* __restrict__ temperature,
                                   int rows_per_seq, int rows, int F, const int32_t* __restrict__ ids, float log_c) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * F) return;
  const int row = i / F;
  const float T = temperature[row / rows_per_seq];
  if (T > 0.f) logits[(int64_t)row * ld + ids[i]] += T * log_c;
}

int launch_sigma_shift(float* logits, int64_t ld, const float* temperature, int rows_per_seq, int rows, int F,
                       const int32_t* ids, float log_c, hipStream_t s) {
  if (rows <= 0) return SSD_OK;
  sigma_shift_kernel<<<(rows * F + 255) / 256, 256, 0, s>>>(logits, ld, temperature, rows_per_seq, rows, F, ids, log_c);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

size_t sample_scratch_bytes(int rows) { return (size_t)rows * kSampleMaxParts * sizeof(ScoreId); }

// scratch: sample_scratch_bytes(rows) of device memory, or null (then every row is one block)
int launch_sample(const float* logits, int64_t ld, const float* temperature, int rows_per_seq, int rows, int V,
                  uint64_t seed, int row_base, int step, int32_t* out, int64_t out_stride, void* scratch, int exact_scan,
                  hipStream_t s) {
  if (rows <= 0) return SSD_OK;
  int parts = 1;
  if (scratch) {
    parts = (2048 + rows - 1) / rows;                                   // about 2048 blocks
    const int by_len = (V + kSelBlock * 4 - 1) / (kSelBlock * 4);       // at least 4 tokens per thread
    parts = parts < by_len ? parts : by_len;
    parts = parts < kSampleMaxParts ? parts : kSampleMaxParts;
    parts = parts < 1 ? 1 : parts;
  }
  // exact_scan: score every token of a sampled row in fp64 instead of pre-selecting in fp32 (a test aid: both give the
  // same token)
  sample_kernel<<<dim3(rows, parts), kSelBlock, 0, s>>>(logits, ld, temperature, rows_per_seq, V, seed, row_base, step, out,
                                                        out_stride, (ScoreId*)scratch, exact_scan);
  SSD_HIP(hipGetLastError());
  if (parts > 1) {
    sample_merge_kernel<<<rows, 64, 0, s>>>((const ScoreId*)scratch, parts, out, out_stride);
    SSD_HIP(hipGetLastError());
  }
  return SSD_OK;
}


int launch_verify(const float* zt, const float* zd, const int32_t* spec, const float* temperature, int B, int K, int V,
                  uint64_t seed, int32_t* accept_len, int32_t* bonus, void* workspace, hipStream_t s) {
  const VerifyWs ws = verify_ws_carve(workspace, B, K);
  const int rows = B * (2 * K + 1);
  // enough blocks to occupy the chip, at least 4096 tokens per part
  int parts = 1024 / rows;
  parts = parts > kVerifyMaxParts ? kVerifyMaxParts : parts;
  while (parts > 1 && V / parts < 4096) --parts;
  parts = parts < 1 ? 1 : parts;
  int parts_b = 512 / B;
  parts_b = parts_b > kVerifyMaxParts ? kVerifyMaxParts : parts_b;
  while (parts_b > 1 && V / parts_b < 4096) --parts_b;
  parts_b = parts_b < 1 ? 1 : parts_b;
  verify_max_kernel<<<dim3(rows, parts), kSelBlock, 0, s>>>(zt, zd, temperature, K, V, ws);
  verify_sum_kernel<<<dim3(rows, parts), kSelBlock, 0, s>>>(zt, zd, temperature, K, V, ws);
  verify_accept_kernel<<<dim3(B, parts_b), kSelBlock, 0, s>>>(zt, zd, spec, temperature, K, V, seed, ws, parts, accept_len, bonus);
  if (zd) {   // without draft logits every sequence is greedy and done
    verify_bonus_kernel<<<dim3(B, parts_b), kSelBlock, 0, s>>>(zt, zd, temperature, K, V, seed, ws);
    verify_bonus_merge_kernel<<<B, 64, 0, s>>>(zd, temperature, parts_b, ws, bonus);
  }
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

// ---- verification for callers that cannot allocate: the workspace is a file-scope device array.  Host code never
// passes the array's name to a kernel (there it is only a host-side stand-in): the device address is looked up once
// per device with hipGetSymbolAddress and kept.
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

size_t verify_static_capacity() { return kStaticScratchBytes; }

int launch_verify_static(const float* zt, const float* zd, const int32_t* spec, const float* temperature, int B, int K, int V,
                         uint64_t seed, int32_t* accept_len, int32_t* bonus, hipStream_t s) {
  const size_t need = verify_workspace_bytes(B, K);
  SSD_CHECK_ARG(need <= kStaticScratchBytes,
                "ssd_verify_static: B = %d, K = %d needs %zu bytes of scratch, the static buffer holds %zu (B (2K+1) <= about 1200)",
                B, K, need, kStaticScratchBytes);
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr_of_device[kMaxDevices] = {};
  int dev = 0;
  SSD_HIP(hipGetDevice(&dev));
  SSD_CHECK_ARG(dev >= 0 && dev < kMaxDevices, "ssd_verify_static: device ordinal %d out of range", dev);
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of_device[dev]) {
      void* p = nullptr;
      SSD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));   // this device's copy of the array (the current device)
      ptr_of_device[dev] = p;
    }
    ptr = ptr_of_device[dev];
  }
  // nothing in the workspace has to start at zero: every word a pass reads was written by an earlier pass of the same call
  return launch_verify(zt, zd, spec, temperature, B, K, V, seed, accept_len, bonus, ptr, s);
}

size_t verify_workspace_bytes(int B, int K) {
  const size_t rows = (size_t)B * (2 * K + 1);
  return verify_ws_align(rows * sizeof(RowStats)) + verify_ws_align(rows * kVerifyMaxParts * sizeof(ScoreId)) +
         verify_ws_align(rows * kVerifyMaxParts * sizeof(double)) + verify_ws_align((size_t)B * kVerifyMaxParts * sizeof(double)) +
         verify_ws_align((size_t)B * kVerifyMaxParts * sizeof(ScoreId)) + verify_ws_align((size_t)B * sizeof(int32_t));
}

}  // namespace ssd
