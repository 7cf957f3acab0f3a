// The fused decode pass (see fused.h): every phase of the decoder runs on all compute units at once inside one
// persistent kernel.
//
// Linear layers.  A workgroup owns whole output-feature tiles over the full reduction dimension, so no partial
// sums cross workgroups and the result does not depend on timing.  Its 8 wavefronts split the reduction dimension;
// each streams its own contiguous run of 1 KiB weight tiles (MFMA 16x16x32 A operands) through a ring of register
// chunks, several KiB in flight per wavefront, and reads the matching activation tiles (B operands: 16 rows x 32
// inputs, written by the producing phase as bf16 head/remainder planes in exactly the lane order the MFMA wants).
// The weight loads of a phase's first chunks are issued BEFORE the workgroup waits at the grid barrier in front of
// that phase: weights depend on nothing, so HBM keeps streaming while the barrier and the small activation exchange
// take their latency.
//
// RMSNorm is split around the linear layer: the producer of the residual stream writes (h * gain) and the
// per-feature-tile sums of h^2; the consumer multiplies its accumulators by the row's 1/rms.
//
// Attention (App. B: every branch row sees the verified trunk up to its fork point plus its own path).  The trunk
// keys of one (sequence, KV head) are shared by all rows and all query heads of the group, so they are scored with
// MFMAs: a unit = (sequence, KV head, group of 8 query tiles, key range); S^T = K Q^T and O^T = V^T P^T keep every
// query row in a fixed lane, so the probabilities feed the second MFMA without leaving their registers (the two
// 16-key score tiles take interleaved key rows so that each lane ends up with 8 consecutive keys).  Values are
// stored transposed in the trunk.  Keys that are private to a row (its own token, its earlier branch tokens, the
// other tokens of an extend) are a handful and go through one wavefront per (row, head).  A second phase merges
// the partial softmaxes.  No mask is ever materialised: a row is (visible trunk length, private suffix length).
#include "fused.h"

namespace ssd {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
// pointers into global memory: loads and stores through these are global_*, never flat_* instructions
typedef __attribute__((address_space(1))) bf16x8 gbf16x8;
typedef __attribute__((address_space(1))) f32x4 gf32x4;
typedef __attribute__((address_space(1))) u32x2 gu32x2;
typedef __attribute__((address_space(1))) float gfloat;
typedef __attribute__((address_space(1))) bf16_t gbf16;

constexpr int MP = kFusedMaxRows;
constexpr int NPA = kFusedActPlanes;
constexpr unsigned kSpinLimit = 4000000u;
constexpr float kLog2e = 1.4426950408889634f;

// Workgroup barrier that waits for LDS traffic only: global loads issued before it stay in flight.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Write-through stores: visible to every other compute unit once the issuing wavefront's vmcnt reaches zero.
__device__ __forceinline__ void st_u64(void* p, uint64_t v) {
  __hip_atomic_store((uint64_t*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_f32(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t pack_f32x2(float a, float b) {
  return (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
}
__device__ __forceinline__ void st_f32x4(float* p, f32x4 v) {
  st_u64(p, pack_f32x2(v[0], v[1]));
  st_u64(p + 2, pack_f32x2(v[2], v[3]));
}
__device__ __forceinline__ uint64_t pack_bf16x4(bf16_t a, bf16_t b, bf16_t c, bf16_t d) {
  return (uint64_t)a | ((uint64_t)b << 16) | ((uint64_t)c << 32) | ((uint64_t)d << 48);
}
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// Optional phase clocks (a measurement aid): [phase][3][workgroup] ticks of the 100 MHz real-time counter at
// phase entry, after the grid barrier, and at the end of the phase's work.
__device__ __forceinline__ void stamp(const FusedParams& p, int ph, int which) {
  if (p.prof && threadIdx.x == 0) p.prof[((int64_t)ph * 3 + which) * p.nwg + blockIdx.x] = __builtin_amdgcn_s_memrealtime();
}

// Offset of element (row m, input k) in a B-operand-ordered activation plane with MT row tiles:
// [k / 32][m / 16][lane = m % 16 + 16 ((k % 32) / 8)][k % 8].
template <int MT>
__device__ __forceinline__ int64_t b_off(int k, int m) {
  return ((int64_t)((k >> 5) * MT + (m >> 4)) * 64 + (m & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7);
}

union Bf8 {
  bf16x8 v;
  uint16_t u[8];
  u32x4 w;
};

// ---------------------------------------------------------------------------------------------- grid barrier
// Two levels: 8 group counters (workgroup g arrives at counter g % 8), the last arrival of a group publishes the
// epoch in that group's flag, every workgroup polls the 8 flags.  Relaxed agent-scope atomics only: data written
// before the arrival went out with write-through stores and s_waitcnt 0.  Every wait is bounded; on expiry the
// error word is set and the workgroup leaves the kernel.
struct Grid {
  unsigned* bar;
  unsigned* err;
  unsigned epoch;
  int persistent;
  int nwg;
  int* dead;   // LDS
};

__device__ __forceinline__ void grid_arrive(Grid& g) {
  if (!g.persistent) return;
  __builtin_amdgcn_s_waitcnt(0);
  wg_barrier();
  ++g.epoch;
  if (threadIdx.x == 0) {
    unsigned grp = blockIdx.x & 7u, per = (unsigned)g.nwg >> 3;
    unsigned old = __hip_atomic_fetch_add(g.bar + 64 * grp, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1 == g.epoch * per)
      __hip_atomic_store(g.bar + 512 + grp, g.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

__device__ __forceinline__ bool grid_wait(Grid& g) {
  if (!g.persistent) return true;
  if (threadIdx.x < 8) {
    unsigned spins = 0;
    while (__hip_atomic_load(g.bar + 512 + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < g.epoch) {
      if (++spins > kSpinLimit) {
        __hip_atomic_store(g.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *g.dead = 1;
        break;
      }
    }
  }
  wg_barrier();
  return *g.dead == 0;
}

// 1/rms of every row from the per-feature-tile partial sums of squares: r_s[m] (LDS).
__device__ __forceinline__ void compute_row_scales(const FusedParams& p, const float* ssq, float* r_s) {
  const int n_tiles = p.d >> 4;
  const int m = threadIdx.x >> 3, part = threadIdx.x & 7;
  float s = 0.f;
  if (m < p.M)
    for (int j = part; j < n_tiles; j += 8) s += ((const gfloat*)ssq)[j * MP + m];
  s += __shfl_xor(s, 1);
  s += __shfl_xor(s, 2);
  s += __shfl_xor(s, 4);
  if (m < p.M && part == 0) r_s[m] = 1.0f / sqrtf(s / (float)p.d + p.eps);
  wg_barrier();
}

// Residual-stream epilogue shared by the embedding, the o-projection and the down-projection: store the new h
// (4 consecutive features n..n+3 of row m per lane), (h * gain) as head/remainder planes for the next linear
// layer, and this feature tile's sum of squares per row.
template <int MT>
__device__ __forceinline__ void resid_store(const FusedParams& p, f32x4 hn, int m, int n, int lane, const bf16_t* gain,
                                            float* h_out, bf16_t* xn_out, float* ssq_out, int tile) {
  const bool ok = m < p.M;
  float s = 0.f;
  if (ok) {
    st_f32x4(h_out + (int64_t)m * p.d + n, hn);
    u32x2 gb = *(const gu32x2*)(gain + n);
    float g[4] = {__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xffff0000u), __uint_as_float(gb.y << 16),
                  __uint_as_float(gb.y & 0xffff0000u)};
    bf16_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float x = hn[i] * g[i];
      hi[i] = f32_to_bf16(x);
      lo[i] = f32_to_bf16(x - bf16_to_f32(hi[i]));
      s += hn[i] * hn[i];
    }
    int64_t off = b_off<MT>(n, m);
    st_u64(xn_out + off, pack_bf16x4(hi[0], hi[1], hi[2], hi[3]));
    st_u64(xn_out + (int64_t)MP * p.d + off, pack_bf16x4(lo[0], lo[1], lo[2], lo[3]));
  }
  s += __shfl_xor(s, 16);
  s += __shfl_xor(s, 32);
  if (ok && lane < 16) st_f32(ssq_out + tile * MP + m, s);
}

// ---------------------------------------------------------------------------------------------- linear layers
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct EpiArgs {
  float* out;          // QKV: [M][ld] raw projections; LOGITS: [M][ld] logits
  int64_t ld;
  const float* h_in;   // RESID
  float* h_out;
  const bf16_t* gain;
  bf16_t* xn_out;
  float* ssq_out;
  bf16_t* act_out;     // SWIGLU
};

template <int AT, int MT, int NP>
struct Chunk {
  bf16x8 a[AT];
  bf16x8 b[MT * NP];
};

// One linear layer over the workgroup's units.  bsrc: activation planes in B-operand order, `bplane` elements apart.
// ssq_in: if not null, row scales are computed into r_s after the barrier (SWIGLU and LOGITS need them).
template <int AT, int MT, int NP, int D, int EPI>
__device__ __forceinline__ bool gemm_phase(const FusedParams& p, const FusedGemm g, const bf16_t* bsrc, int64_t bplane,
                                           const EpiArgs& e, Grid& grid, bool do_wait, f32x4* red, float* r_s,
                                           const float* ssq_in, int ph) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int KTW = g.KTW;
  const int n_my = (int)blockIdx.x < g.n_units ? (g.n_units - 1 - (int)blockIdx.x) / p.nwg + 1 : 0;
  const int n_chunks = n_my * KTW;
  Chunk<AT, MT, NP> ring[D];

  // chunk c = (unit blockIdx.x + n * grid, k-tile i of this wavefront); the load cursors advance one chunk at a time
  const gbf16x8* a_next = (const gbf16x8*)(g.w + (((int64_t)blockIdx.x * kFusedWaves + wave) * KTW * AT) * 512 + lane * 8);
  const int64_t a_unit_jump = ((int64_t)p.nwg * kFusedWaves - 1) * KTW * AT * 64;   // in 16-byte vectors, added at a unit's end
  int a_i = 0;
  auto load_a = [&](Chunk<AT, MT, NP>& ck) {
#pragma unroll
    for (int j = 0; j < AT; ++j) ck.a[j] = __builtin_nontemporal_load(a_next + j * 64);
    a_next += AT * 64;
    if (++a_i == KTW) { a_i = 0; a_next += a_unit_jump; }
  };
  const gbf16x8* b_first = (const gbf16x8*)(bsrc + ((int64_t)(wave * KTW) * MT * 64 + lane) * 8);
  const int64_t bplane_v = bplane / 8;
  int b_i = 0;
  auto load_b = [&](Chunk<AT, MT, NP>& ck) {
    const gbf16x8* bp = b_first + (int64_t)b_i * MT * 64;
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int pl = 0; pl < NP; ++pl) ck.b[t * NP + pl] = bp[pl * bplane_v + t * 64];
    if (++b_i == KTW) b_i = 0;
  };

  // weights of the first chunks go out before the barrier: they depend on nothing
  if (n_chunks > 0) {
#pragma unroll
    for (int s = 0; s < D - 1; ++s) load_a(ring[s]);
  }
  if (do_wait && !grid_wait(grid)) return false;
  stamp(p, ph, 1);
  if (n_chunks > 0) {
#pragma unroll
    for (int s = 0; s < D - 1; ++s) load_b(ring[s]);
  }
  if (ssq_in) compute_row_scales(p, ssq_in, r_s);

  f32x4 acc[AT][MT];
#pragma unroll
  for (int j = 0; j < AT; ++j)
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[j][t] = (f32x4){0.f, 0.f, 0.f, 0.f};

  auto mfma_chunk = [&](const Chunk<AT, MT, NP>& ck) {
#pragma unroll
    for (int j = 0; j < AT; ++j)
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int pl = 0; pl < NP; ++pl)
          acc[j][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ck.a[j], ck.b[t * NP + pl], acc[j][t], 0, 0, 0);
  };

  // End of a unit: sum the 8 wavefronts' partial tiles in LDS and run the epilogue.
  auto finish_unit = [&](int unit) {
#pragma unroll
    for (int j = 0; j < AT; ++j)
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        red[(wave * (AT * MT) + j * MT + t) * 64 + lane] = acc[j][t];
        acc[j][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
    wg_barrier();
    constexpr int NOUT = EPI == EPI_SWIGLU ? 2 * MT : AT * MT;
    for (int idx = wave; idx < NOUT; idx += kFusedWaves) {
      const int j = idx / MT, t = idx - j * MT;
      f32x4 v = red[(j * MT + t) * 64 + lane];
#pragma unroll
      for (int w = 1; w < kFusedWaves; ++w) v += red[(w * (AT * MT) + j * MT + t) * 64 + lane];
      const int m = t * 16 + (lane & 15);
      const int f4 = (lane >> 4) * 4;
      if (EPI == EPI_QKV) {
        const int n = (unit * AT + j) * 16 + f4;
        if (m < p.M) st_f32x4(e.out + (int64_t)m * e.ld + n, v);
      } else if (EPI == EPI_RESID) {
        const int tile = unit * AT + j;
        const int n = tile * 16 + f4;
        f32x4 ho = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (m < p.M) ho = *(const gf32x4*)(e.h_in + (int64_t)m * p.d + n);
        resid_store<MT>(p, ho + v, m, n, lane, e.gain, e.h_out, e.xn_out, e.ssq_out, tile);
      } else if (EPI == EPI_SWIGLU) {
        // tiles 0,1 of the unit are gate, 2,3 the matching up tiles; idx = (gate tile j, row tile t)
        f32x4 u = red[((j + 2) * MT + t) * 64 + lane];
#pragma unroll
        for (int w = 1; w < kFusedWaves; ++w) u += red[(w * (AT * MT) + (j + 2) * MT + t) * 64 + lane];
        if (m < p.M) {
          const float rs = r_s[m];
          bf16_t hi[4], lo[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float gg = v[i] * rs, uu = u[i] * rs;
            float a = gg / (1.0f + __expf(-gg)) * uu;
            hi[i] = f32_to_bf16(a);
            lo[i] = f32_to_bf16(a - bf16_to_f32(hi[i]));
          }
          const int k = unit * 32 + j * 16 + f4;    // input index of the down-projection
          int64_t off = b_off<MT>(k, m);
          st_u64(e.act_out + off, pack_bf16x4(hi[0], hi[1], hi[2], hi[3]));
          if (NPA == 2) st_u64(e.act_out + (int64_t)MP * p.ffn + off, pack_bf16x4(lo[0], lo[1], lo[2], lo[3]));
        }
      } else {
        const int tile = unit * AT + j;
        const int n = tile * 16 + f4;
        if (m < p.M && tile < g.NT) {
          const float rs = r_s[m];
          *(gf32x4*)(e.out + (int64_t)m * e.ld + n) = v * rs;
        }
      }
    }
    // Loads and stores share one counter and may complete out of order with respect to each other: drain it here,
    // once per unit, so that the chunk waits in the streaming loop stay exact.
    __builtin_amdgcn_s_waitcnt(0);
    wg_barrier();
  };

  // The host guarantees KTW % D == 0: a unit ends only at the end of a group of D chunks, and every load inside
  // the steady loop is unconditional (the compiler then counts outstanding loads exactly).
  const int n_outer = n_chunks / D;
  int c_i = 0, c_unit = blockIdx.x;
  for (int q = 0; q + 1 < n_outer; ++q) {
#pragma unroll
    for (int s = 0; s < D; ++s) {
      load_a(ring[(s + D - 1) % D]);
      load_b(ring[(s + D - 1) % D]);
      mfma_chunk(ring[s]);
    }
    c_i += D;
    if (c_i == KTW) {
      c_i = 0;
      finish_unit(c_unit);
      c_unit += p.nwg;
    }
  }
  if (n_outer > 0) {
    load_a(ring[D - 1]);
    load_b(ring[D - 1]);
#pragma unroll
    for (int s = 0; s < D; ++s) mfma_chunk(ring[s]);
    finish_unit(c_unit);
  }
  return true;
}

// ---------------------------------------------------------------------------------------------- attention
__device__ __forceinline__ int trunk_visible(const RowDesc& r, int m, int R) {
  // stored trunk keys the row sees; the tokens of this very pass are handled as fresh keys
  return r.is_branch ? r.vis : r.vis - 1 - (m % R);
}

// Rotary embedding of element d (0..63) of a head, given the element and its partner (d ^ 32).
__device__ __forceinline__ float rope_elem(float own, float partner, float c, float s, int d) {
  return d < 32 ? own * c - partner * s : own * c + partner * s;
}

// Trunk unit: all query rows of (sequence b, KV head hk) in q tiles qg*8 .. qg*8+7 (one per wavefront) against the
// stored trunk keys [s KPU, (s+1) KPU).
template <int NPQ, int NPP>
__device__ __forceinline__ void attn_trunk_unit(const FusedParams& p, const FusedLayer& L, const float* qkv, int unit,
                                                const float* r_s, float* part_o, float* part_ml) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int per = p.B * p.Hkv * p.NS;
  const int qg = unit / per;
  int rem = unit - qg * per;
  const int hk = rem % p.Hkv;
  rem /= p.Hkv;
  const int s = rem % p.NS, b = rem / p.NS;
  const int qt = qg * 8 + wave;
  if (qt >= p.QT) return;
  const int RG = p.R * p.G;
  const int qr = qt * 16 + (lane & 15);
  const bool vq = qr < RG;
  const int qrc = vq ? qr : RG - 1;
  const int m = b * p.R + qrc / p.G;
  const int hq = hk * p.G + qrc % p.G;
  const int g4 = lane >> 4;
  const RowDesc rd = p.rows[m];
  const int tv = vq ? trunk_visible(rd, m, p.R) : 0;
  int tvmax = tv;
  for (int o = 32; o > 0; o >>= 1) tvmax = max(tvmax, __shfl_xor(tvmax, o));
  const int kb0 = s * p.KPU;
  const int kend = min(kb0 + p.KPU, tvmax);

  // Q operand: dims g4*8..+7 (k-step 0) and 32+g4*8..+7 (k-step 1) of this lane's query row, rotated and scaled
  Bf8 qh[2], ql[2];
  {
    const float* qp = qkv + (int64_t)m * p.qkvd + hq * 64 + g4 * 8;
    f32x4 a0 = *(const gf32x4*)qp, a1 = *(const gf32x4*)(qp + 4);
    f32x4 b0 = *(const gf32x4*)(qp + 32), b1 = *(const gf32x4*)(qp + 36);
    const float* cs = p.cos_sin + ((int64_t)m * 32 + g4 * 8) * 2;
    f32x4 c0 = *(const gf32x4*)cs, c1 = *(const gf32x4*)(cs + 4), c2 = *(const gf32x4*)(cs + 8), c3 = *(const gf32x4*)(cs + 12);
    float a[8] = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
    float bb[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
    float cc[16] = {c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3],
                    c2[0], c2[1], c2[2], c2[3], c3[0], c3[1], c3[2], c3[3]};
    const float scale = r_s[m] * 0.125f * kLog2e;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float c = cc[2 * i], sn = cc[2 * i + 1];
      float x0 = (a[i] * c - bb[i] * sn) * scale, x1 = (bb[i] * c + a[i] * sn) * scale;
      qh[0].u[i] = f32_to_bf16(x0);
      qh[1].u[i] = f32_to_bf16(x1);
      ql[0].u[i] = f32_to_bf16(x0 - bf16_to_f32(qh[0].u[i]));
      ql[1].u[i] = f32_to_bf16(x1 - bf16_to_f32(qh[1].u[i]));
    }
  }

  f32x4 acc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) acc[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;
  const bf16_t* kbase = L.trunk_k + ((int64_t)b * p.max_trunk * p.Hkv + hk) * 64 + g4 * 8;
  const bf16_t* vbase = L.trunk_vt + (((int64_t)b * p.Hkv + hk) * 64 + (lane & 15)) * p.vt_stride + g4 * 8;
  const int krow = ((lane & 15) >> 2) * 8 + (lane & 3);   // key row of this lane inside a 32-key block (tile 0)

  for (int kb = kb0; kb < kend; kb += 32) {
    f32x4 S[2];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      int key = min(kb + krow + tile * 4, p.max_trunk - 1);
      const bf16_t* kp = kbase + (int64_t)key * p.Hkv * 64;
      bf16x8 k0 = *(const gbf16x8*)kp, k1 = *(const gbf16x8*)(kp + 32);
      f32x4 sacc = (f32x4){0.f, 0.f, 0.f, 0.f};
      sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qh[0].v, sacc, 0, 0, 0);
      sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qh[1].v, sacc, 0, 0, 0);
      if (NPQ == 2) {
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, ql[0].v, sacc, 0, 0, 0);
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, ql[1].v, sacc, 0, 0, 0);
      }
      S[tile] = sacc;
    }
    // this lane: query row lane & 15, keys kb + g4*8 + {0..3} (tile 0) and + {4..7} (tile 1)
    float sv[8];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int key = kb + g4 * 8 + i;
      float x = i < 4 ? S[0][i] : S[1][i - 4];
      sv[i] = key < tv ? x : -INFINITY;
      mx = fmaxf(mx, sv[i]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float corr = exp2_fast(m_run - m_use);
    Bf8 ph, pl;
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float pe = exp2_fast(sv[i] - m_use);
      psum += pe;
      ph.u[i] = f32_to_bf16(pe);
      pl.u[i] = f32_to_bf16(pe - bf16_to_f32(ph.u[i]));
    }
    l_run = l_run * corr + psum;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      bf16x8 vt = *(const gbf16x8*)(vbase + (int64_t)dt * 16 * p.vt_stride + kb);
      acc[dt] = acc[dt] * corr;
      acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, ph.v, acc[dt], 0, 0, 0);
      if (NPP == 2) acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt, pl.v, acc[dt], 0, 0, 0);
    }
  }
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (vq) {
    const int64_t pb = ((int64_t)(b * p.Hkv + hk) * (p.NS + 1) + s) * (p.QG * 128) + qr;
    if (g4 == 0) st_u64(part_ml + pb * 2, pack_f32x2(m_run, l_run));
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) st_f32x4(part_o + pb * 64 + dt * 16 + g4 * 4, acc[dt]);
  }
}

__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Pair unit: one wavefront per (row, query head), lane = head dimension.  Keys that exist only in this pass or
// only for this row: the row's own token, its stored private suffix (branch rows), the earlier tokens of the same
// extend (extend rows).  Also appends the row's K/V to its suffix slot or trunk position (first head of a group).
__device__ __forceinline__ void attn_pair_unit(const FusedParams& p, const FusedLayer& L, const float* qkv, int unit,
                                               const float* r_s, float* part_o, float* part_ml) {
  const int d = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pair = unit * kFusedWaves + wave;
  if (pair >= p.M * p.Hq) return;
  const int m = pair / p.Hq, hq = pair - m * p.Hq;
  const int hk = hq / p.G, gq = hq - hk * p.G;
  const RowDesc rd = p.rows[m];
  const int b = rd.seq;
  const int t_self = m - b * p.R;
  const int i = d & 31;

  auto rotated = [&](int row, int col0) -> float {   // rotary embedding at `row`'s position of head columns col0..+63
    const gfloat* src = (const gfloat*)qkv + (int64_t)row * p.qkvd + col0;
    const gfloat* cs = (const gfloat*)p.cos_sin + ((int64_t)row * 32 + i) * 2;
    return rope_elem(src[d], src[d ^ 32], cs[0], cs[1], d) * r_s[row];
  };
  const float q = rotated(m, hq * 64) * (0.125f * kLog2e);
  // this row's own key and value, rounded to the KV storage type like every other key
  const bf16_t k_self = f32_to_bf16(rotated(m, p.qd + hk * 64));
  const bf16_t v_self = f32_to_bf16(((const gfloat*)qkv)[(int64_t)m * p.qkvd + p.qd + p.kvd + hk * 64 + d] * r_s[m]);

  const int nk = rd.is_branch ? rd.suffix_len : t_self + 1;
  float m_run = -INFINITY, l_run = 0.f, o = 0.f;
  for (int j = 0; j < nk; ++j) {
    float kj, vj;
    if (j == nk - 1) {
      kj = bf16_to_f32(k_self);
      vj = bf16_to_f32(v_self);
    } else if (rd.is_branch) {
      int64_t off = (((int64_t)m * p.suffix_cap + j) * p.Hkv + hk) * 64 + d;
      kj = bf16_to_f32(((const gbf16*)L.suffix_k)[off]);
      vj = bf16_to_f32(((const gbf16*)L.suffix_v)[off]);
    } else {
      int row = b * p.R + j;
      kj = bf16_to_f32(f32_to_bf16(rotated(row, p.qd + hk * 64)));
      vj = bf16_to_f32(f32_to_bf16(((const gfloat*)qkv)[(int64_t)row * p.qkvd + p.qd + p.kvd + hk * 64 + d] * r_s[row]));
    }
    const float sc = wave_sum(q * kj);
    const float m_new = fmaxf(m_run, sc);
    const float corr = exp2_fast(m_run - m_new);
    const float pe = exp2_fast(sc - m_new);
    l_run = l_run * corr + pe;
    o = o * corr + pe * vj;
    m_run = m_new;
  }
  const int qr = t_self * p.G + gq;
  const int64_t pb = ((int64_t)(b * p.Hkv + hk) * (p.NS + 1) + p.NS) * (p.QG * 128) + qr;
  st_f32(part_o + pb * 64 + d, o);
  if (d == 0) st_u64(part_ml + pb * 2, pack_f32x2(m_run, l_run));
  if (gq == 0) {
    if (rd.is_branch) {
      int64_t off = (((int64_t)m * p.suffix_cap + rd.kv_slot) * p.Hkv + hk) * 64 + d;
      ((gbf16*)L.suffix_k)[off] = k_self;
      ((gbf16*)L.suffix_v)[off] = v_self;
    } else {
      ((gbf16*)L.trunk_k)[(((int64_t)b * p.max_trunk + rd.kv_slot) * p.Hkv + hk) * 64 + d] = k_self;
      ((gbf16*)L.trunk_vt)[(((int64_t)b * p.Hkv + hk) * 64 + d) * p.vt_stride + rd.kv_slot] = v_self;
    }
  }
}

// Combine unit: one wavefront per (row, query head) merges the partial softmaxes of the key splits the row sees
// and of its fresh keys, and writes the attention output as head/remainder planes for the o-projection.
template <int MT>
__device__ __forceinline__ void attn_combine_unit(const FusedParams& p, int unit, const float* part_o,
                                                  const float* part_ml, bf16_t* att_out) {
  const int d = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pair = unit * kFusedWaves + wave;
  if (pair >= p.M * p.Hq) return;
  const int m = pair / p.Hq, hq = pair - m * p.Hq;
  const int hk = hq / p.G, gq = hq - hk * p.G;
  const RowDesc rd = p.rows[m];
  const int b = rd.seq;
  const int qr = (m - b * p.R) * p.G + gq;
  const int tv = trunk_visible(rd, m, p.R);
  const int nsv = min(p.NS, (tv + p.KPU - 1) / p.KPU);
  const int64_t pb0 = ((int64_t)(b * p.Hkv + hk) * (p.NS + 1)) * (p.QG * 128) + qr;
  float m_run = -INFINITY, l_run = 0.f, o = 0.f;
  for (int j = 0; j <= nsv; ++j) {
    const int s = j < nsv ? j : p.NS;
    const int64_t pb = pb0 + (int64_t)s * (p.QG * 128);
    const float ms = ((const gfloat*)part_ml)[pb * 2], ls = ((const gfloat*)part_ml)[pb * 2 + 1];
    const float os = ((const gfloat*)part_o)[pb * 64 + d];
    const float m_new = fmaxf(m_run, ms);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float c1 = exp2_fast(m_run - m_use), c2 = exp2_fast(ms - m_use);
    l_run = l_run * c1 + ls * c2;
    o = o * c1 + os * c2;
    m_run = m_new;
  }
  const float x = o / l_run;
  const bf16_t hi = f32_to_bf16(x);
  const bf16_t lo = f32_to_bf16(x - bf16_to_f32(hi));
  // lanes d, d+1, d+2, d+3 -> one 8-byte store per plane from lane d (d % 4 == 0)
  uint32_t w = (uint32_t)hi | ((uint32_t)lo << 16);
  uint32_t w1 = __shfl_down(w, 1), w2 = __shfl_down(w, 2), w3 = __shfl_down(w, 3);
  if ((d & 3) == 0) {
    const int k = hq * 64 + d;
    const int64_t off = b_off<MT>(k, m);
    st_u64(att_out + off, pack_bf16x4((bf16_t)w, (bf16_t)w1, (bf16_t)w2, (bf16_t)w3));
    st_u64(att_out + (int64_t)MP * p.qd + off,
           pack_bf16x4((bf16_t)(w >> 16), (bf16_t)(w1 >> 16), (bf16_t)(w2 >> 16), (bf16_t)(w3 >> 16)));
  }
}

// ---------------------------------------------------------------------------------------------- the kernel
// Register chunks in flight per wavefront.  DEEP needs the k-tiles per wavefront of every linear layer to be a
// multiple of 8 (one feature tile per unit) / 4 (four per unit); the shallow set needs multiples of 2.
template <int MT, bool DEEP> struct Depth {
  static constexpr int a1 = !DEEP ? 2 : (MT == 3 ? 4 : 8);   // one feature tile per unit
  static constexpr int a4 = !DEEP ? 2 : (MT == 3 ? 2 : 4);   // four feature tiles per unit
};

template <int MT, bool DEEP>
__global__ __launch_bounds__(kFusedThreads) void fused_kernel(FusedParams p, int first, int last, int persistent) {
  extern __shared__ f32x4 red[];
  __shared__ float r_s[64];
  __shared__ int dead;
  if (threadIdx.x == 0) dead = 0;
  wg_barrier();
  Grid grid{p.bar, p.err, 0u, persistent, p.nwg, &dead};
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t h_stride = (int64_t)MP * p.d;
  const int64_t ssq_stride = (int64_t)(p.d >> 4) * MP;
  const int lm_phase = fused_last_phase(p.L);

  for (int ph = first; ph <= last; ++ph) {
    const bool do_wait = persistent && ph > first;
    stamp(p, ph, 0);
    if (ph == 0) {
      // ---- embedding gather: residual stream version 0
      const FusedLayer L0 = p.layers[0];
      for (int u = blockIdx.x; u < (p.d >> 4); u += p.nwg) {
        if (wave < MT) {
          const int m = wave * 16 + (lane & 15);
          const int n = u * 16 + (lane >> 4) * 4;
          int tok = p.tokens[min(m, p.M - 1)];
          tok = tok < 0 ? 0 : (tok >= p.V ? p.V - 1 : tok);
          u32x2 eb = *(const gu32x2*)(p.embed + (int64_t)tok * p.d + n);
          f32x4 hn = (f32x4){__uint_as_float(eb.x << 16), __uint_as_float(eb.x & 0xffff0000u),
                             __uint_as_float(eb.y << 16), __uint_as_float(eb.y & 0xffff0000u)};
          resid_store<MT>(p, hn, m, n, lane, L0.attn_norm, p.h, p.xn, p.ssq, u);
        }
      }
    } else if (ph == lm_phase) {
      const int v = 2 * p.L;
      EpiArgs e{};
      e.out = p.logits;
      e.ld = p.logits_ld;
      // final-norm hidden states go out first: they need only the row scales
      if (do_wait && !grid_wait(grid)) return;
      stamp(p, ph, 1);
      compute_row_scales(p, p.ssq + v * ssq_stride, r_s);
      if (p.hidden) {
        const float* hv = p.h + v * h_stride;
        for (int m = blockIdx.x; m < p.M; m += p.nwg)
          for (int c = threadIdx.x; c < p.d; c += kFusedThreads)
            p.hidden[(int64_t)m * p.hidden_ld + c] = hv[(int64_t)m * p.d + c] * bf16_to_f32(p.final_norm[c]) * r_s[m];
      }
      if (p.logits &&
          !gemm_phase<kAtLm, MT, 2, Depth<MT, DEEP>::a4, EPI_LOGITS>(p, p.lm, p.xn + v * 2 * h_stride, h_stride, e, grid, false,
                                                              red, r_s, nullptr, ph))
        return;
    } else {
      const int l = (ph - 1) / 6, sub = (ph - 1) % 6;
      const FusedLayer L = p.layers[l];
      float* qkv = p.qkv + (int64_t)l * MP * p.qkvd;
      bf16_t* att = p.att + (int64_t)l * 2 * MP * p.qd;
      bf16_t* act = p.act + (int64_t)l * NPA * MP * p.ffn;
      float* part_o = p.part_o + (int64_t)l * p.part_layer_stride * 64;
      float* part_ml = p.part_ml + (int64_t)l * p.part_layer_stride * 2;
      if (sub == 0) {
        EpiArgs e{};
        e.out = qkv;
        e.ld = p.qkvd;
        if (!gemm_phase<kAtQkv, MT, 2, Depth<MT, DEEP>::a1, EPI_QKV>(p, L.qkv, p.xn + (int64_t)(2 * l) * 2 * h_stride, h_stride, e,
                                                              grid, do_wait, red, r_s, nullptr, ph))
          return;
      } else if (sub == 1) {
        if (do_wait && !grid_wait(grid)) return;
        stamp(p, ph, 1);
        compute_row_scales(p, p.ssq + (int64_t)(2 * l) * ssq_stride, r_s);
        const int n_units = p.n_trunk_units + p.n_pair_units;
        for (int u = blockIdx.x; u < n_units; u += p.nwg) {
          if (u < p.n_trunk_units) attn_trunk_unit<2, 2>(p, L, qkv, u, r_s, part_o, part_ml);
          else attn_pair_unit(p, L, qkv, u - p.n_trunk_units, r_s, part_o, part_ml);
        }
      } else if (sub == 2) {
        if (do_wait && !grid_wait(grid)) return;
        stamp(p, ph, 1);
        for (int u = blockIdx.x; u < p.n_pair_units; u += p.nwg) attn_combine_unit<MT>(p, u, part_o, part_ml, att);
      } else if (sub == 3) {
        const int v = 2 * l + 1;
        EpiArgs e{};
        e.h_in = p.h + (int64_t)(v - 1) * h_stride;
        e.h_out = p.h + (int64_t)v * h_stride;
        e.gain = L.mlp_norm;
        e.xn_out = p.xn + (int64_t)v * 2 * h_stride;
        e.ssq_out = p.ssq + (int64_t)v * ssq_stride;
        if (!gemm_phase<kAtO, MT, 2, Depth<MT, DEEP>::a1, EPI_RESID>(p, L.o, att, (int64_t)MP * p.qd, e, grid, do_wait, red, r_s,
                                                              nullptr, ph))
          return;
      } else if (sub == 4) {
        const int v = 2 * l + 1;
        EpiArgs e{};
        e.act_out = act;
        if (!gemm_phase<kAtGu, MT, 2, Depth<MT, DEEP>::a4, EPI_SWIGLU>(p, L.gu, p.xn + (int64_t)v * 2 * h_stride, h_stride, e, grid,
                                                                do_wait, red, r_s, p.ssq + (int64_t)v * ssq_stride, ph))
          return;
      } else {
        const int v = 2 * l + 2;
        EpiArgs e{};
        e.h_in = p.h + (int64_t)(v - 1) * h_stride;
        e.h_out = p.h + (int64_t)v * h_stride;
        e.gain = l + 1 < p.L ? p.layers[l + 1].attn_norm : p.final_norm;
        e.xn_out = p.xn + (int64_t)v * 2 * h_stride;
        e.ssq_out = p.ssq + (int64_t)v * ssq_stride;
        if (!gemm_phase<kAtDown, MT, NPA, Depth<MT, DEEP>::a1, EPI_RESID>(p, L.down, act, (int64_t)MP * p.ffn, e, grid, do_wait,
                                                                     red, r_s, nullptr, ph))
          return;
      }
    }
    stamp(p, ph, 2);
    if (ph < last) grid_arrive(grid);
  }
}

// ---------------------------------------------------------------------------------------------- set-up kernels
__global__ void retile_stream_kernel(const bf16_t* __restrict__ src0, int rows0, const bf16_t* __restrict__ src1, int rows1,
                                     const bf16_t* __restrict__ src2, int rows2, int mode, int AT, int Kd, int n_units,
                                     bf16_t* __restrict__ dst) {
  const int KTW = Kd / 32 / kFusedWaves;
  const int64_t total = (int64_t)n_units * kFusedWaves * KTW * AT * 64;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int lane = (int)(idx & 63);
  int64_t tile = idx >> 6;
  const int j = (int)(tile % AT);
  tile /= AT;
  const int i = (int)(tile % KTW);
  tile /= KTW;
  const int w = (int)(tile % kFusedWaves);
  const int64_t u = tile / kFusedWaves;
  const int kt = w * KTW + i;
  const bf16_t* src = nullptr;
  int64_t row = 0;
  if (mode == 0) {
    int64_t n = (u * AT + j) * 16 + (lane & 15);
    if (n < rows0) { src = src0; row = n; }
    else if (n < (int64_t)rows0 + rows1) { src = src1; row = n - rows0; }
    else if (n < (int64_t)rows0 + rows1 + rows2) { src = src2; row = n - rows0 - rows1; }
  } else {
    int64_t n = (2 * u + (j & 1)) * 16 + (lane & 15);
    if (n < rows0) { src = j < 2 ? src0 : src1; row = n; }
  }
  u32x4 v = (u32x4){0u, 0u, 0u, 0u};
  if (src) v = *(const u32x4*)(src + row * Kd + kt * 32 + (lane >> 4) * 8);
  *(u32x4*)(dst + idx * 8) = v;
}

__global__ void copy_v_transposed_kernel(bf16_t* trunk_vt, const bf16_t* src, int len, int Hkv, int vt_stride, int64_t total) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // over [B][len][Hkv][64]
  if (idx >= total) return;
  int d = (int)(idx & 63);
  int64_t r = idx >> 6;
  int hk = (int)(r % Hkv);
  r /= Hkv;
  int pos = (int)(r % len);
  int64_t b = r / len;
  trunk_vt[((b * Hkv + hk) * 64 + d) * vt_stride + pos] = src[idx];
}

template <int MT, bool DEEP>
int launch_mt(const FusedParams& p, int first, int last, int persistent, hipStream_t s) {
  const size_t lds = 96 * 1024;   // reduction tiles (<= 8 wavefronts x 12 tiles x 1 KiB); also keeps one workgroup per CU
  static bool configured = false;
  if (!configured) {
    SSD_HIP(hipFuncSetAttribute((const void*)fused_kernel<MT, DEEP>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    configured = true;
  }
  if (persistent) {
    fused_kernel<MT, DEEP><<<p.nwg, kFusedThreads, lds, s>>>(p, first, last, 1);
    SSD_HIP(hipGetLastError());
  } else {
    for (int ph = first; ph <= last; ++ph) {
      fused_kernel<MT, DEEP><<<p.nwg, kFusedThreads, lds, s>>>(p, ph, ph, 0);
      SSD_HIP(hipGetLastError());
    }
  }
  return SSD_OK;
}

}  // namespace

int64_t stream_order_elems(int N, int Kd, int AT) {
  int64_t nt = (N + 15) / 16;
  int64_t units = (nt + AT - 1) / AT;
  return units * AT * 16 * (int64_t)Kd;
}

int launch_retile_stream(const bf16_t* src0, int rows0, const bf16_t* src1, int rows1, const bf16_t* src2, int rows2,
                         int mode, int AT, int Kd, bf16_t* dst, hipStream_t s) {
  SSD_CHECK_ARG(Kd % 256 == 0, "fused path: reduction dimension %d must be a multiple of 256", Kd);
  SSD_CHECK_ARG(mode == 0 || (AT == 4 && rows0 == rows1 && rows0 % 32 == 0), "gate/up interleave needs AT = 4 and equal heights");
  int64_t nt = mode == 0 ? ((int64_t)rows0 + rows1 + rows2 + 15) / 16 : (int64_t)2 * (rows0 / 16);
  int n_units = (int)((nt + AT - 1) / AT);
  int64_t total = (int64_t)n_units * AT * (Kd / 32) * 64;
  retile_stream_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(src0, rows0, src1, rows1, src2, rows2, mode, AT, Kd,
                                                                       n_units, dst);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_copy_v_transposed(bf16_t* trunk_vt, const bf16_t* src, int B, int len, int Hkv, int vt_stride, hipStream_t s) {
  int64_t total = (int64_t)B * len * Hkv * 64;
  if (total == 0) return SSD_OK;
  copy_v_transposed_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(trunk_vt, src, len, Hkv, vt_stride, total);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

bool fused_supported(const Dims& d, int max_rows) {
  return d.dtype == SSD_BF16 && d.head_dim == 64 && max_rows <= kFusedMaxRows && d.d_model % 512 == 0 &&
         d.q_dim() % 512 == 0 && d.d_ffn % 512 == 0 && d.kv_dim() % 16 == 0 && d.vocab % 16 == 0 &&
         d.n_q_heads % d.n_kv_heads == 0;
}

int fused_grid_size(int* out) {
  int dev = 0;
  SSD_HIP(hipGetDevice(&dev));
  int cus = 0;
  SSD_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  cus -= cus % 8;
  if (cus < 8) {
    set_error("fused path needs at least 8 compute units");
    return SSD_EINVAL;
  }
  *out = cus;
  return SSD_OK;
}

int launch_fused(const FusedParams& p, int first, int last, int persistent, hipStream_t s) {
  SSD_CHECK_ARG(p.M >= 1 && p.M <= kFusedMaxRows, "fused pass of %d rows (1..%d supported)", p.M, kFusedMaxRows);
  SSD_CHECK_ARG(p.nwg >= 8 && p.nwg % 8 == 0, "fused grid of %d workgroups must be a multiple of 8", p.nwg);
  SSD_CHECK_ARG(p.KPU >= 32 && p.KPU % 32 == 0 && p.NS >= 1 && p.QG >= 1 && p.QT <= p.QG * 8, "bad attention split");
  SSD_CHECK_ARG(first >= 0 && last <= fused_last_phase(p.L) && first <= last, "bad phase range");
  const int mt = (p.M + 15) / 16;
  const int k_d = p.d / 256, k_q = p.qd / 256, k_f = p.ffn / 256;
  SSD_CHECK_ARG(k_d % 2 == 0 && k_q % 2 == 0 && k_f % 2 == 0, "fused pass: d_model, q_dim and d_ffn must be multiples of 512");
  const bool deep = k_d % 8 == 0 && k_q % 8 == 0 && k_f % 8 == 0;
  if (deep) {
    if (mt == 1) return launch_mt<1, true>(p, first, last, persistent, s);
    if (mt == 2) return launch_mt<2, true>(p, first, last, persistent, s);
    return launch_mt<3, true>(p, first, last, persistent, s);
  }
  if (mt == 1) return launch_mt<1, false>(p, first, last, persistent, s);
  if (mt == 2) return launch_mt<2, false>(p, first, last, persistent, s);
  return launch_mt<3, false>(p, first, last, persistent, s);
}

}  // namespace ssd
