// The fused decode pass (see fused.h): every phase of the decoder runs on all compute units at once inside one
// persistent kernel.
//
// Linear layers.  A workgroup owns whole output-feature tiles ("owner computes"): over the full reduction dimension
// for the qkv, gate/up and LM-head projections, over one of 2 or 4 k-slices of it for the o and down projections,
// whose slices hand their partial tiles to slice 0 through memory; slice 0 adds them in slice order, so the result
// does not depend on timing.  The 8 wavefronts of a workgroup split its reduction range; each streams its own
// contiguous run of 1 KiB weight tiles (MFMA 16x16x32 A operands, fp16) and reads the matching activation tiles (B
// operands: 16 rows x 32 inputs, written by the producing phase as fp16 head/remainder planes in exactly the lane
// order the MFMA wants).  Two loop shapes: where a workgroup has at most one unit (qkv, o, down) ALL its weight
// tiles are requested before it waits at the grid barrier in front of the phase; gate/up and the LM head stream
// weights and activations together through a ring of register chunks whose first chunks go out before the barrier.
// Weights depend on nothing, so HBM keeps streaming while the barrier and the activation exchange take their latency.
// One exchange needs less than the grid: an attention unit reads the projections of its KV head's group only, so the
// qkv units of a group announce themselves in a line of flags that the group's attention units poll (group_wait), and
// no grid barrier stands between a layer's qkv phase and its attention phase.
//
// RMSNorm is split around the linear layer: the producer of the residual stream writes (h * gain) and the
// per-feature-tile sums of h^2; the consumer multiplies its accumulators by the row's 1/rms.
//
// Attention (App. B: every branch row sees the verified trunk up to its fork point plus its own path).  The trunk
// keys of one (sequence, KV head) are shared by all rows and all query heads of the group, so they are scored with
// MFMAs: a unit = (sequence, KV head, one 16-row query tile of rows x group heads, key split); S^T = K Q^T and
// O^T = V^T P^T keep every query row in a fixed lane, so the probabilities feed the second MFMA without leaving their
// registers (the two 16-key score tiles take interleaved key rows so that each lane ends up with 8 consecutive
// keys).  Values are stored transposed in the trunk.  The keys computed in this very pass (a branch row's own token
// and its earlier branch tokens, the other tokens of an extend) are rotated and staged in LDS by the unit and go
// through the same MFMAs under a per-row visibility test; the unit appends them to the KV store afterwards.  With
// one key split the unit writes the final output; with several, every unit stores its partial softmax and counts its
// arrival, and the unit that arrives last of a tile's splits merges them in split order (wide passes: a merge phase).
// No mask is ever materialised: a row is (visible trunk length, private suffix length).
#include <type_traits>
#include <vector>

#include "fused.h"

namespace ssd {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
// pointers into global memory: loads and stores through these are global_*, never flat_* instructions
typedef __attribute__((address_space(1))) bf16x8 gbf16x8;
typedef __attribute__((address_space(1))) f32x4 gf32x4;
typedef __attribute__((address_space(1))) u32x2 gu32x2;
typedef __attribute__((address_space(1))) float gfloat;
typedef __attribute__((address_space(1))) bf16_t gbf16;

// 16-bit planes per activation tensor: 2 = head + remainder, 1 = the head alone.  xn: (h * gain) feeding qkv, gate/up
// and the LM head; att: attention output feeding the o-projection; act: SwiGLU output feeding the down-projection:
// these three meet the weights and are fp16 (head alone: 11 significant bits; with the remainder about 22).  q, p: the
// rotated queries and the softmax probabilities inside the attention unit, which meet the bf16 keys and values and are
// bf16 (8 bits, or about 16 with the remainder).
template <int X, int T, int C, int Q, int P>
struct Planes {
  static constexpr int xn = X, att = T, act = C, q = Q, p = P;
};
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
// Partial tiles of a K-split are their own "ready" flag: a word that holds kFixEmpty (a NaN pattern no sum of
// products produces) has not been written in this launch.  The reader takes the tile with agent-scope loads (coherent
// across the XCDs) and writes kFixEmpty back.
constexpr unsigned kFixEmpty = 0xffffffffu;
__device__ __forceinline__ f32x4 ld_f32x4_coherent(const float* p) {
  const uint64_t a = __hip_atomic_load((const uint64_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const uint64_t b = __hip_atomic_load((const uint64_t*)p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return (f32x4){__uint_as_float((unsigned)a), __uint_as_float((unsigned)(a >> 32)), __uint_as_float((unsigned)b),
                 __uint_as_float((unsigned)(b >> 32))};
}
__device__ __forceinline__ bool fix_ready(f32x4 v) {
  return __float_as_uint(v[0]) != kFixEmpty && __float_as_uint(v[1]) != kFixEmpty && __float_as_uint(v[2]) != kFixEmpty &&
         __float_as_uint(v[3]) != kFixEmpty;
}
__device__ __forceinline__ f32x4 fix_empty() {
  const float e = __uint_as_float(kFixEmpty);
  return (f32x4){e, e, e, e};
}
// A plain 16-byte store the compiler does not see as a memory operation.  With a store pending, the compiler's waits
// for loads degrade to "wait for everything", which would empty the weight pipeline at every unit of the LM head.
// Hidden, the store only makes a later counted wait err on the safe side: loads complete in order among themselves,
// so "at most N operations outstanding" still implies that every load older than the N youngest has arrived.
// (the s_nop: a store of more than 8 bytes must not be followed at once by a VALU write of its data registers, a
// hazard the compiler covers for its own stores and cannot see inside this one)
__device__ __forceinline__ void st_f32x4_uncounted(float* p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off\n\ts_nop 0" : : "v"(p), "v"(v));
}
// Thread coordinates read afresh where they are called: everything derived from them (row and tile indices, LDS and
// global addresses) is then local to the phase that computes it.  Derived from the kernel-wide threadIdx they would be
// hoisted out of the phase loop, stay live through every phase and be spilled where registers are short.
struct ThreadIds { int tid, lane, wave; };
__device__ __forceinline__ ThreadIds fresh_thread_ids() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return ThreadIds{t, t & 63, __builtin_amdgcn_readfirstlane(t >> 6)};
}
// The lane index, recomputed where it is called (the compiler can neither hoist nor remember the result).
__device__ __forceinline__ int fresh_lane_id() {
  int l;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
  return l;
}
__device__ __forceinline__ uint64_t pack_bf16x4(bf16_t a, bf16_t b, bf16_t c, bf16_t d) {
  return (uint64_t)a | ((uint64_t)b << 16) | ((uint64_t)c << 32) | ((uint64_t)d << 48);
}
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
// fp32 -> bf16, round to nearest even, on the conversion unit gfx950 has for it (v_cvt_pk_bf16_f32): the softmax and the
// head/remainder splits convert thousands of values per phase, and the integer sequence costs ~8 VALU instructions each
__device__ __forceinline__ bf16_t to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// The linear layers multiply in fp16 x fp16 -> fp32.  An activation that travels as ONE 16-bit plane keeps 11 significant
// bits in fp16 where bf16 keeps 8: through 16 layers that is 2.5e-3 instead of 2e-2 between the hidden states and a
// float64 reference (measured on 384-row passes), for the same bytes and the same MFMA rate.  The weights are converted
// once, when the stream-order layout is built (exact for |w| >= 2^-14; smaller ones round to fp16 subnormals, absolute
// error <= 2^-25); activations saturate at the fp16 range.  Keys, values, queries and probabilities stay bf16.
__device__ __forceinline__ uint16_t to_f16(float x) {
  const _Float16 h = (_Float16)fminf(fmaxf(x, -65504.0f), 65504.0f);
  return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float f16_to_f32(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ __forceinline__ f32x4 mfma16_f16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma32_f16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Optional phase clocks (a measurement aid): [phase][slot][workgroup] ticks of the 100 MHz real-time counter; slot 0
// phase entry, 1 after the grid barrier, 2 end of the phase's work, 3.. probes inside a phase.
__device__ __forceinline__ void stamp(const FusedParams& p, int ph, int which) {
  // (launches of more workgroups than the grid of the persistent kernel - the attention, merge and hidden-state launches
  // of a wide pass - record their first p.nwg workgroups: the table has p.nwg columns)
  if (p.prof && threadIdx.x == 0 && (int)blockIdx.x < p.nwg)
    p.prof[((int64_t)ph * kFusedClockSlots + which) * p.nwg + blockIdx.x] = __builtin_amdgcn_s_memrealtime();
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
// Two levels: kBarGroups group counters (workgroup g arrives at counter g % kBarGroups), the last arrival of a group
// publishes the epoch in that group's flag, every workgroup polls all the flags.  Relaxed agent-scope atomics only: data written
// before the arrival went out with write-through stores and s_waitcnt 0.  Every wait is bounded; on expiry the
// error word is set and the workgroup leaves the kernel.
constexpr int kBarGroups = 2;        // a power of two that divides the grid; measured per layer of the 1B shape:
                                     // 1 group 51.7 us, 2 50.5, 4 50.9, 8 51.3, 16 52.2, 32 53.8 (more flags to poll
                                     // against fewer arrivals queueing at one counter)
constexpr int kBarFlags = 1024;      // barrier words: group counters at 32 g (a cache line each), flags at 1024 + g,
constexpr int kBarEpochWord = 1100;  // the epoch here
struct Grid {
  unsigned* bar;
  unsigned* err;
  unsigned epoch;
  int persistent;
  int nwg;
  int* dead;   // LDS
  unsigned spin_limit;   // polls a bounded wait may take before it gives up
};

__device__ __forceinline__ void grid_arrive(Grid& g) {
  if (!g.persistent) return;
  __builtin_amdgcn_s_waitcnt(0);
  wg_barrier();
  ++g.epoch;
  if (threadIdx.x == 0) {
    unsigned grp = blockIdx.x & (unsigned)(kBarGroups - 1), per = (unsigned)g.nwg / kBarGroups;
    unsigned old = __hip_atomic_fetch_add(g.bar + 32 * grp, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1 == g.epoch * per)
      __hip_atomic_store(g.bar + kBarFlags + grp, g.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

__device__ __forceinline__ bool grid_wait(Grid& g) {
  if (!g.persistent) return true;
  if (threadIdx.x < kBarGroups) {
    unsigned spins = 0;
    // (compared as a signed difference: the epoch counts on across launches and may wrap)
    while ((int)(__hip_atomic_load(g.bar + kBarFlags + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - g.epoch) < 0) {
      if (++spins > g.spin_limit) {
        __hip_atomic_store(g.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        *g.dead = 1;
        break;
      }
      // no pause between polls: each one already takes a memory round trip, and only kBarGroups lanes of a
      // workgroup poll (measured: 0.3 us per layer faster than with a 64-cycle sleep; several polls in flight: no gain)
    }
  }
  wg_barrier();
  return *g.dead == 0;
}

// Attention needs less than the whole grid behind it: an attention unit of KV head g reads the projections of that
// head's group only (its query heads, its key head, its value head), which `n` workgroups own in the qkv phase.  Each of
// them, once its stores have left, writes the current barrier number into its word of the group's line of flags
// (one 64-byte line per layer and group); the unit polls that one line.  The grid barrier between the qkv and the
// attention phase is gone with it; workgroups without a unit pass straight on.  The barrier number is the same on
// both sides (nobody arrives at a grid barrier in between) and differs from launch to launch.
__device__ __forceinline__ bool group_wait(Grid& g, const unsigned* line, int n) {
  if (!g.persistent) return true;
  if ((int)threadIdx.x < n) {
    unsigned spins = 0;
    while (__hip_atomic_load(line + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != g.epoch) {
      if (++spins > g.spin_limit) {
        __hip_atomic_store(g.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        *g.dead = 1;
        break;
      }
    }
  }
  wg_barrier();
  return *g.dead == 0;
}

// 1/rms of every row from the per-feature-tile partial sums of squares: r_s[m] (LDS).  MP: row capacity of the workspace.
template <int MP>
__device__ __forceinline__ void compute_row_scales(const FusedParams& p, const float* ssq, float* r_s) {
  const int n_tiles = p.d >> 4;
  const int m = threadIdx.x >> 3, part = threadIdx.x & 7;
  const gfloat* src = (const gfloat*)ssq + (m < p.M ? m : 0);
  float s = 0.f;
  // 16 independent loads at a time: a chain of dependent loads would cost a memory latency each
  for (int j0 = part; j0 < n_tiles; j0 += 128) {
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      int j = j0 + 8 * i;
      v[i] = src[(j < n_tiles ? j : j0) * MP];
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) s += j0 + 8 * i < n_tiles ? v[i] : 0.f;
  }
  s += __shfl_xor(s, 1);
  s += __shfl_xor(s, 2);
  s += __shfl_xor(s, 4);
  if (m < p.M && part == 0) r_s[m] = 1.0f / sqrtf(s / (float)p.d + p.eps);
  wg_barrier();
}

// Residual-stream epilogue shared by the embedding, the o-projection and the down-projection: store the new h
// (4 consecutive features n..n+3 of row m per lane), (h * gain) as fp16 head/remainder planes for the next linear
// layer, and this feature tile's sum of squares per row.
template <int MT, int MP, int NPX>
__device__ __forceinline__ void resid_store(const FusedParams& p, f32x4 hn, int m, int n, int lane, u32x2 gb,
                                            float* h_out, bf16_t* xn_out, float* ssq_out, int tile) {
  const bool ok = m < p.M;
  float s = 0.f;
  if (ok) {
    st_f32x4(h_out + (int64_t)m * p.d + n, hn);
    float g[4] = {__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xffff0000u), __uint_as_float(gb.y << 16),
                  __uint_as_float(gb.y & 0xffff0000u)};
    bf16_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float x = hn[i] * g[i];
      hi[i] = to_f16(x);
      lo[i] = to_f16(x - f16_to_f32(hi[i]));
      s += hn[i] * hn[i];
    }
    int64_t off = b_off<MT>(n, m);
    st_u64(xn_out + off, pack_bf16x4(hi[0], hi[1], hi[2], hi[3]));
    if (NPX == 2) st_u64(xn_out + (int64_t)MP * p.d + off, pack_bf16x4(lo[0], lo[1], lo[2], lo[3]));
  }
  s += __shfl_xor(s, 16);
  s += __shfl_xor(s, 32);
  if (ok && lane < 16) st_f32(ssq_out + tile * MP + m, s);
}

// ---------------------------------------------------------------------------------------------- linear layers
enum { FE_QKV = 0, FE_RESID = 1, FE_SWIGLU = 2, FE_LOGITS = 3 };

struct EpiArgs {
  float* out;          // QKV: [M][ld] raw projections; LOGITS: [M][ld] logits
  int64_t ld;
  const float* h_in;   // RESID
  float* h_out;
  const bf16_t* gain;
  bf16_t* xn_out;
  float* ssq_out;
  bf16_t* act_out;     // SWIGLU
  float* fix_buf;      // K-split: [tile group][slice][tile][64 lanes][4] partial tiles of this phase instance
};

template <int AT, int MT, int NP>
struct Chunk {
  bf16x8 a[AT];
  bf16x8 b[MT * NP];
};

// One linear layer over the workgroup's units.  bsrc: activation planes in B-operand order, `bplane` elements apart.
// ssq_in: if not null, row scales are computed into r_s after the barrier (SWIGLU and LOGITS need them).
// AT = 2 serves the qkv, o and down projections (epilogue FE_QKV / FE_RESID), AT = 4 the gate/up projection and the
// LM head (FE_SWIGLU / FE_LOGITS).  The epilogue kind is a run-time argument so that each of the two streaming loops
// exists once in the kernel: its code has to stay resident in the instruction cache across the layers.
// MP: row capacity of the workspace; NPX / NPC: planes of the (h * gain) / SwiGLU outputs the epilogues write.
template <int AT, int MT, int NP, int D, bool PRE, int MP, int NPX, int NPC>
__device__ __forceinline__ bool gemm_phase(const FusedParams& p, const FusedGemm g, const bf16_t* bsrc, int64_t bplane,
                                           const int EPI, const EpiArgs& e, Grid& grid, bool do_wait, f32x4* red, float* r_s,
                                           const float* ssq_in, int ph, int my_unit) {
  // my_unit: the unit of this workgroup in a phase of at most one unit per workgroup (PRE), or -1
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int KTW = g.KTW;
  // K-split (g.KS > 1, at most one unit per workgroup): unit u = (feature-tile group u / KS, k-slice u % KS)
  const int KS = g.KS, ks = KS > 1 ? (my_unit < 0 ? 0 : my_unit % KS) : 0;
  const gbf16x8* b_first = (const gbf16x8*)(bsrc + ((int64_t)((ks * kFusedWaves + wave) * KTW) * MT * 64 + lane) * 8);
  const int64_t bplane_v = bplane / 8;

  f32x4 acc[AT][MT];
#pragma unroll
  for (int j = 0; j < AT; ++j)
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[j][t] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // End of a unit: sum the 8 wavefronts' partial tiles in LDS and run the epilogue.
  auto finish_unit = [&](int unit) {
    // The lane index of the epilogue is read afresh here: addresses derived from the function-wide `lane` would be
    // kept across the streaming loop, where registers are short, spilled, and their reloads (memory loads like any
    // other) would make the compiler wait for the whole weight pipeline at every unit.
    const int lane = fresh_lane_id();
    // the residual-stream tile and the gains this wavefront's epilogue will want: requested now, so that they arrive
    // under the LDS reduction and the K-split fix-up instead of costing a memory latency at the very end
    f32x4 h_pre = (f32x4){0.f, 0.f, 0.f, 0.f};
    u32x2 gain_pre = (u32x2){0u, 0u};
    if (AT <= 2 && EPI == FE_RESID && wave < AT * MT && ks == 0) {
      const int j = wave / MT, t = wave - j * MT;
      const int tile = (KS > 1 ? unit / KS : unit) * AT + j;
      const int m = t * 16 + (lane & 15), n = tile * 16 + (lane >> 4) * 4;
      if (m < p.M) h_pre = *(const gf32x4*)(e.h_in + (int64_t)m * p.d + n);
      gain_pre = *(const gu32x2*)(e.gain + n);
    }
#pragma unroll
    for (int j = 0; j < AT; ++j)
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        red[(wave * (AT * MT) + j * MT + t) * 64 + lane] = acc[j][t];
        acc[j][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
    wg_barrier();
    const int NOUT = EPI == FE_SWIGLU ? 2 * MT : AT * MT;
    const int tg = KS > 1 ? unit / KS : unit;     // feature-tile group of the unit
    if (KS > 1 && ks > 0) {
      // K-split, slices 1..: publish the reduced tiles.  The partial-tile buffer holds kFixEmpty words between
      // launches, so the data are their own "ready" flag and no counter or extra round trip is needed.
      float* fix = e.fix_buf + ((int64_t)tg * KS) * (AT * MT) * 256;
      for (int idx = wave; idx < AT * MT; idx += kFusedWaves) {
        f32x4 v = red[idx * 64 + lane];
#pragma unroll
        for (int w = 1; w < kFusedWaves; ++w) v += red[(w * (AT * MT) + idx) * 64 + lane];
        st_f32x4(fix + ((int64_t)ks * (AT * MT) + idx) * 256 + lane * 4, v);
      }
      __builtin_amdgcn_s_waitcnt(0);
      wg_barrier();
      return;
    }
    for (int idx = wave; idx < NOUT; idx += kFusedWaves) {
      const int j = idx / MT, t = idx - j * MT;
      f32x4 v = red[(j * MT + t) * 64 + lane];
#pragma unroll
      for (int w = 1; w < kFusedWaves; ++w) v += red[(w * (AT * MT) + j * MT + t) * 64 + lane];
      if (KS > 1) {
        // Ordered fix-up: slice 0 polls the other slices' tiles until no word is kFixEmpty, adds them in slice order
        // (the result does not depend on timing) and puts kFixEmpty back for the next launch.
        float* fix = e.fix_buf + ((int64_t)tg * KS) * (AT * MT) * 256 + (int64_t)idx * 256 + lane * 4;
        f32x4 pv[kFusedMaxSlices - 1];
        unsigned pending = (1u << (KS - 1)) - 1u, spins = 0;
        while (pending) {
#pragma unroll
          for (int q = 0; q < kFusedMaxSlices - 1; ++q)
            if (pending >> q & 1u) pv[q] = ld_f32x4_coherent(fix + (int64_t)(q + 1) * (AT * MT) * 256);
#pragma unroll
          for (int q = 0; q < kFusedMaxSlices - 1; ++q)
            if ((pending >> q & 1u) && fix_ready(pv[q])) pending &= ~(1u << q);
          if (pending && ++spins > grid.spin_limit) {
            __hip_atomic_store(grid.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            *grid.dead = 1;
            break;
          }
        }
#pragma unroll
        for (int q = 0; q < kFusedMaxSlices - 1; ++q)
          if (q + 1 < KS) {
            v += pv[q];
            st_f32x4(fix + (int64_t)(q + 1) * (AT * MT) * 256, fix_empty());
          }
      }
      const int m = t * 16 + (lane & 15);
      const int f4 = (lane >> 4) * 4;
      if (AT <= 2 && EPI == FE_QKV) {
        const int n = (tg * AT + j) * 16 + f4;
        if (m < p.M) st_f32x4(e.out + (int64_t)m * e.ld + n, v);
      } else if (AT <= 2 && EPI == FE_RESID) {
        const int tile = tg * AT + j;
        const int n = tile * 16 + f4;
        resid_store<MT, MP, NPX>(p, h_pre + v, m, n, lane, gain_pre, e.h_out, e.xn_out, e.ssq_out, tile);   // idx == wave here
      } else if (AT == 4 && EPI == FE_SWIGLU) {
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
            hi[i] = to_f16(a);
            lo[i] = to_f16(a - f16_to_f32(hi[i]));
          }
          const int k = unit * 32 + j * 16 + f4;    // input index of the down-projection
          int64_t off = b_off<MT>(k, m);
          st_u64(e.act_out + off, pack_bf16x4(hi[0], hi[1], hi[2], hi[3]));
          if (NPC == 2) st_u64(e.act_out + (int64_t)MP * p.ffn + off, pack_bf16x4(lo[0], lo[1], lo[2], lo[3]));
        }
      } else if (AT == 4) {
        const int tile = unit * AT + j;
        const int n = tile * 16 + f4;
        if (m < p.M && tile < g.NT) {
          const float rs = r_s[m];
          st_f32x4_uncounted(e.out + (int64_t)m * e.ld + n, v * rs);
        }
      }
    }
    // Loads and stores share one counter and may complete out of order with respect to each other: drain it here,
    // once per unit, so that the chunk waits in the streaming loop stay exact.  The LM head, the one phase with several
    // units per workgroup, must not drain (the next unit's weights are already in flight): its stores are not counted
    // (see st_f32x4_uncounted) and complete under the next unit; the drain before the grid barrier covers them.
    if (EPI != FE_LOGITS) __builtin_amdgcn_s_waitcnt(0);
    wg_barrier();
  };


  if constexpr (PRE) {
    // ---- at most one unit per workgroup (the host checks n_units <= grid): ALL of the wavefront's weight tiles are
    // requested before the workgroup waits at the barrier, so the weight stream of the phase runs under the barrier
    // latency, the activation fetch and the row scales; after the barrier only the activation tiles (L2) are loaded,
    // through a short ring.  KTW is a run-time value: one fully unrolled instance per supported value, so that every
    // register index is static and the compiler counts outstanding loads exactly.
    if (my_unit < 0 || my_unit >= g.n_units) {
      if (do_wait && !grid_wait(grid)) return false;
      stamp(p, ph, 1);
      if (ssq_in) compute_row_scales<MP>(p, ssq_in, r_s);
      return true;
    }
    constexpr int KMAX = 16 / AT;   // most k-tiles per wavefront and unit (the host checks)
    const gbf16x8* a_base = (const gbf16x8*)(g.w + (((int64_t)my_unit * kFusedWaves + wave) * KTW * AT) * 512 + lane * 8);
    bf16x8 a[KMAX][AT];
#pragma unroll
    for (int i = 0; i < KMAX; ++i)
      if (i < KTW) {
#pragma unroll
        for (int j = 0; j < AT; ++j) a[i][j] = __builtin_nontemporal_load(a_base + (i * AT + j) * 64);
      }
    if (do_wait && !grid_wait(grid)) return false;
    stamp(p, ph, 1);
    // Activation tiles.  Every workgroup reads the whole activation matrix of its k-range, and all of them the same
    // lines at the same time: this L2-to-CU traffic, not the weight stream, is what limits these phases, so rows
    // beyond M (the padding of the last 16-row tile) are not fetched at all.
    // (their lanes re-read row 0 of their k-group, a line that is fetched anyway; an unconditional load keeps the
    // compiler's count of outstanding loads exact, and those rows' results are never stored)
    int row_fix[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) row_fix[t] = t * 16 + (lane & 15) < p.M ? 0 : -(lane & 15);
    auto load_b = [&](bf16x8* dst, int c) {
      const gbf16x8* bp = b_first + (int64_t)c * MT * 64;
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) dst[t * NP + pl] = bp[pl * bplane_v + t * 64 + row_fix[t]];
    };
    // the activation tiles of KC chunks through a ring of DB, straight-line code with static register indices
    auto run = [&](auto kc_tag) {
      constexpr int KC = decltype(kc_tag)::value;
      constexpr int DB = KC < 4 ? KC : 4;
      bf16x8 b[DB][MT * NP];
#pragma unroll
      for (int c = 0; c < DB - 1; ++c) load_b(b[c], c);
#pragma unroll
      for (int c = 0; c < KC; ++c) {
        if (c + DB - 1 < KC) load_b(b[(c + DB - 1) % DB], c + DB - 1);
#pragma unroll
        for (int j = 0; j < AT; ++j)
#pragma unroll
          for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int pl = 0; pl < NP; ++pl)
              acc[j][t] = mfma16_f16(a[c][j], b[c % DB][t * NP + pl], acc[j][t]);
      }
    };
    if (KTW == 2) run(std::integral_constant<int, 2>());
    else if (KTW == 4) run(std::integral_constant<int, 4>());
    else run(std::integral_constant<int, 8>());
    stamp(p, ph, 3);
    if (ssq_in) compute_row_scales<MP>(p, ssq_in, r_s);   // for the next phase (qkv -> attention)
    stamp(p, ph, 4);
    finish_unit(my_unit);
    stamp(p, ph, 5);
    return true;
  } else {
    // ---- any number of units per workgroup (the LM head): weights and activations travel together through a ring
    // of D register chunks
    const int n_my = (int)blockIdx.x < g.n_units ? (g.n_units - 1 - (int)blockIdx.x) / p.nwg + 1 : 0;
    const int n_chunks = n_my * KTW;
    Chunk<AT, MT, NP> ring[D];
    // chunk c = (unit blockIdx.x + n * grid, k-tile i of this wavefront); the load cursors advance one chunk at a time
    const gbf16x8* a_next = (const gbf16x8*)(g.w + (((int64_t)blockIdx.x * kFusedWaves + wave) * KTW * AT) * 512 + lane * 8);
    const int64_t a_unit_jump = ((int64_t)p.nwg * kFusedWaves - 1) * KTW * AT * 64;   // in 16-byte vectors, at a unit's end
    int a_i = 0;
    auto load_a = [&](Chunk<AT, MT, NP>& ck) {
#pragma unroll
      for (int j = 0; j < AT; ++j) ck.a[j] = __builtin_nontemporal_load(a_next + j * 64);
      a_next += AT * 64;
      if (++a_i == KTW) { a_i = 0; a_next += a_unit_jump; }
    };
    int b_i = 0;
    int row_fix[MT];   // rows beyond M (padding of the last row tile) are not fetched: their lanes re-read row 0
#pragma unroll
    for (int t = 0; t < MT; ++t) row_fix[t] = t * 16 + (lane & 15) < p.M ? 0 : -(lane & 15);
    auto load_b = [&](Chunk<AT, MT, NP>& ck) {
      const gbf16x8* bp = b_first + (int64_t)b_i * MT * 64;
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) ck.b[t * NP + pl] = bp[pl * bplane_v + t * 64 + row_fix[t]];
      if (++b_i == KTW) b_i = 0;
    };
    auto mfma_chunk = [&](const Chunk<AT, MT, NP>& ck) {
#pragma unroll
      for (int j = 0; j < AT; ++j)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
          for (int pl = 0; pl < NP; ++pl)
            acc[j][t] = mfma16_f16(ck.a[j], ck.b[t * NP + pl], acc[j][t]);
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
    if (ssq_in) compute_row_scales<MP>(p, ssq_in, r_s);
    stamp(p, ph, 3);
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
      stamp(p, ph, 4);
      load_a(ring[D - 1]);
      load_b(ring[D - 1]);
#pragma unroll
      for (int s = 0; s < D; ++s) mfma_chunk(ring[s]);
      stamp(p, ph, 5);
      finish_unit(c_unit);
    }
    return true;
  }
}

// ---------------------------------------------------------------------------------------------- attention
// Reductions over the four 16-lane rows of a wavefront (lanes l, l^16, l^32, l^48 hold values of one query row) with
// the row-swap instructions of gfx950: a swap of a register with itself leaves "mine" in one result and "my
// partner's" in the other, a few cycles instead of a trip through the LDS crossbar.
__device__ __forceinline__ float max_over_rows(float x) {
  const unsigned u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned v = __float_as_uint(fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1])));
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float sum_over_rows(float x) {
  const unsigned u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned v = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
__device__ __forceinline__ int trunk_visible(const RowDesc& r, int m, int R) {
  // stored trunk keys the row sees; the tokens of this very pass are handled as fresh keys
  return r.is_branch ? r.vis : r.vis - 1 - (m % R);
}

struct OnlineSoftmax {
  float m_run, l_run;   // running maximum (base-2 exponent) and this lane's share of the running sum
  f32x4 acc[4];         // O^T: dims dt*16 + (lane>>4)*4 + r of query row lane & 15
};

// Online-softmax update with the block's masked scores sv (this lane's 8 keys) and their maximum mx.  The running
// accumulators are rescaled only when some row's maximum moved (a wavefront-uniform test): after the first blocks it
// rarely does.
template <int NPP>
__device__ __forceinline__ void softmax_update(OnlineSoftmax& st, const float sv[8], float mx, const bf16x8 vt[4]) {
  mx = max_over_rows(mx);
  const float m_new = fmaxf(st.m_run, mx);
  const float m_use = m_new == -INFINITY ? 0.f : m_new;
  if (__any(m_new != st.m_run)) {
    const float corr = exp2_fast(st.m_run - m_use);
    st.l_run *= corr;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) st.acc[dt] = st.acc[dt] * corr;
    st.m_run = m_new;
  }
  Bf8 ph, pl;
  float psum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float pe = exp2_fast(sv[i] - m_use);
    psum += pe;
    ph.u[i] = to_bf16(pe);
    pl.u[i] = to_bf16(pe - bf16_to_f32(ph.u[i]));
  }
  st.l_run += psum;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    st.acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt[dt], ph.v, st.acc[dt], 0, 0, 0);
    if (NPP == 2) st.acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt[dt], pl.v, st.acc[dt], 0, 0, 0);
  }
}


// One 32-key block: scores S[tile][r] of this lane's query row against keys (lane>>4)*8 + tile*4 + r of the block,
// `vis` = visibility of those 8 keys, vt[dt] = V^T operands of the block.
template <int NPP>
__device__ __forceinline__ void softmax_block(OnlineSoftmax& st, const f32x4 S[2], const bool vis[8], const bf16x8 vt[4]) {
  float sv[8];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float x = i < 4 ? S[0][i] : S[1][i - 4];
    sv[i] = vis[i] ? x : -INFINITY;
    mx = fmaxf(mx, sv[i]);
  }
  softmax_update<NPP>(st, sv, mx, vt);
}

template <int NPQ>
__device__ __forceinline__ f32x4 score_tile(bf16x8 k0, bf16x8 k1, const Bf8 qh[2], const Bf8 ql[2]) {
  f32x4 s = (f32x4){0.f, 0.f, 0.f, 0.f};
  s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qh[0].v, s, 0, 0, 0);
  s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qh[1].v, s, 0, 0, 0);
  if (NPQ == 2) {
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, ql[0].v, s, 0, 0, 0);
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, ql[1].v, s, 0, 0, 0);
  }
  return s;
}

// Attention unit = (sequence b, KV head hk, 16-row query tile qt, key split s).  A query tile holds 16 / G whole
// rows with all G query heads of the group.  The 8 wavefronts take the 32-key blocks of the unit round-robin:
// first the stored trunk keys of the split, then (split 0 only) the blocks of "fresh" keys: keys that exist only in
// this pass or only for one row.  Branch rows: fresh key f = (row of the tile f / SL, slot f % SL), the row's
// stored private suffix followed by its own token, visible to that row alone.  Extend rows: fresh key f = token f
// of this pass, visible to rows f and later.  All 512 threads stage the fresh K rows and V^T columns in LDS (and
// append the new K/V to the suffix or the trunk).  A dependent global load costs more than a microsecond here, so
// every load whose address is pure index arithmetic (row descriptors, the query tile, the first trunk blocks, the
// fresh-key sources) is issued up front; loop counts come from the host's bound on the visible trunk, the true
// visibility only masks.  The 8 partial softmaxes meet in LDS; with one split the result goes straight to the
// o-projection's operand planes, otherwise to the partial buffers that the last unit of the tile to arrive merges.
// SM: the unit that arrives last of a tile's key splits merges them (a kernel of its own for passes with several splits:
// compiled into the one-split kernel, the merge costs its linear layers 1 % through their register allocation).
template <int MT, int MP, int NPQ, int NPP, int NPT, bool PG, bool SM>
__device__ __forceinline__ bool attn_unit(const FusedParams& p, const FusedLayer& L, const float* qkv, int unit,
                                          const float* r_s, f32x4* lds, bf16_t* att_out, float* part_o, float* part_ml,
                                          unsigned* arrivals, int ph, Grid* wait_on, const unsigned* group_flags) {
  const ThreadIds ids = fresh_thread_ids();
  const int lane = ids.lane, wave = ids.wave;
  const int li = lane & 15, g4 = lane >> 4;
  const int hk = unit % p.Hkv;
  int rem = unit / p.Hkv;
  const int qt = rem % p.QT;
  rem /= p.QT;
  const int s = rem % p.NS, b = rem / p.NS;
  const int g_log = 31 - __builtin_clz(p.G), sl_log = p.SL == 8 ? 3 : 4;   // G and SL are powers of two
  const int RG = p.R << g_log;
  const int qr = qt * 16 + li;
  const bool vq = qr < RG;
  const int qrc = vq ? qr : RG - 1;
  const int rloc = qrc >> g_log;           // row of the sequence
  const int m = b * p.R + rloc;
  const int hq = hk * p.G + (qrc & (p.G - 1));
  const bool is_branch = p.is_branch != 0;
  const gfloat* gq = (const gfloat*)qkv;
  const gfloat* gcs = (const gfloat*)p.cos_sin;

  // ---- issue: the first trunk blocks of this wavefront (block counts from the host's bound)
  const int kb0 = s * p.KPU;
  const int kend_ub = min(kb0 + p.KPU, p.tv_ub);
  const int n_tb = kend_ub > kb0 ? (kend_ub - kb0 + 31) >> 5 : 0;
  const int n_mine = n_tb > wave ? (n_tb - wave + kFusedWaves - 1) / kFusedWaves : 0;
  const int rpt = 16 >> g_log;                                // rows per query tile
  const int n_fresh_keys = is_branch ? rpt << sl_log : p.R;
  const int n_fb = s == 0 ? (n_fresh_keys + 31) >> 5 : 0;
  const int krow = (li >> 2) * 8 + (li & 3);                  // key of this lane's A-operand row in a block (tile 0)
  // trunk K [B][Hkv][vt_stride][64]; trunk V^T [B][Hkv][vt_stride / 32][64 dims][32 keys]: a 32-key block of one head is
  // 4 KiB of contiguous memory in both, so every operand load covers whole cache lines
  // PG (paged trunk, App. B "PagedAttention"): block j of sequence b is page p.pages[b][j] of a pool shared by all
  // sequences, a page = the same 4 KiB per head and operand as a block of the contiguous layouts.  Lane i of a wavefront
  // fetches the page of the wavefront's i-th block up front (one load), so the block loop itself stays free of
  // dependent loads; entries behind a sequence's allocation name page 0, which exists and holds zeros.
  const int64_t head0 = PG ? 0 : ((int64_t)(b * p.Hkv + hk) * p.vt_stride) * 64;
  const gbf16* kbase = (const gbf16*)L.trunk_k + head0 + g4 * 8;
  const gbf16* vbase = (const gbf16*)L.trunk_vt + head0 + li * 32 + g4 * 8;
  int pgs = 0;
  if constexpr (PG) pgs = p.pages[(int64_t)b * p.page_stride + min((kb0 >> 5) + wave + kFusedWaves * lane, p.page_stride - 1)];
  struct TrunkBlock {
    bf16x8 k[2][2];
    bf16x8 vt[4];
  };
  constexpr int RING = 2;
  TrunkBlock ring[RING];
  auto load_trunk = [&](TrunkBlock& tb, int i) {   // i-th block of this wavefront, clamped to its last one
    const int ic = max(min(i, n_mine - 1), 0);
    const int blk = wave + kFusedWaves * ic;
    const int kb = min(kb0 + blk * 32, p.vt_stride - 32);
    const int64_t bo = PG ? ((int64_t)__builtin_amdgcn_readlane(pgs, ic) * p.Hkv + hk) * 2048 : (int64_t)kb * 64;
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      const gbf16* kp = kbase + bo + (krow + tile * 4) * 64;
      tb.k[tile][0] = *(const gbf16x8*)kp;
      tb.k[tile][1] = *(const gbf16x8*)(kp + 32);
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) tb.vt[dt] = *(const gbf16x8*)(vbase + bo + dt * 16 * 32);
  };
#pragma unroll
  for (int i = 0; i < RING; ++i) load_trunk(ring[i], i);   // unconditional (a wavefront without blocks re-reads block 0)
  // The stored keys do not depend on the phase before: the first unit of a workgroup requests its ring ahead of the
  // grid barrier.
  if (wait_on) {
    // the projections of this KV head's group (group_flags: one line of flags per group), or the whole grid
    if (!(group_flags ? group_wait(*wait_on, group_flags + hk * 16, p.qkv_ug) : grid_wait(*wait_on))) return false;
    stamp(p, ph, 1);
  }
  stamp(p, ph, 3);

  // ---- issue: row descriptor, raw query tile
  const RowDesc rd = p.rows[m];
  const gfloat* qp = gq + (int64_t)m * p.qkvd + hq * 64 + g4 * 8;
  const f32x4 qa0 = *(const gf32x4*)qp, qa1 = *(const gf32x4*)(qp + 4);
  const f32x4 qb0 = *(const gf32x4*)(qp + 32), qb1 = *(const gf32x4*)(qp + 36);
  const gfloat* qcs = gcs + ((int64_t)m * 32 + g4 * 8) * 2;
  const f32x4 qc0 = *(const gf32x4*)qcs, qc1 = *(const gf32x4*)(qcs + 4), qc2 = *(const gf32x4*)(qcs + 8), qc3 = *(const gf32x4*)(qcs + 12);

  // ---- issue: sources of the fresh key this thread stages (item = key f, rotary quad / 8-dim group q8)
  struct Fresh {
    int f, q8, m_o;
    bool valid, stored;
    u32x2 k_lo, k_hi;      // stored: 4 + 4 key elements
    bf16x8 v;              // stored: 8 value elements
    f32x4 a, bb, c0, c1, v0, v1;   // computed: raw projections and rotary table
  };
  int fresh_slot = 0;    // extend rows: trunk position the fresh key is appended at
  Fresh fr[1];
  const int nf8 = n_fb * 32 * 8;   // at most 512: one item per thread
#pragma unroll
  for (int t = 0; t < 1; ++t) {
    Fresh& x = fr[t];
    const int it = threadIdx.x + t * kFusedThreads;
    x.f = it >> 3;
    x.q8 = it & 7;
    x.valid = false;
    x.stored = false;
    x.m_o = b * p.R;
    if (it < nf8) {
      if (is_branch) {
        const int rt = qt * rpt + (x.f >> sl_log), j = x.f & (p.SL - 1);
        x.m_o = b * p.R + min(rt, p.R - 1);
        x.valid = rt < p.R && j < p.suffix_len;
        x.stored = j < p.suffix_len - 1;
        if (x.valid && x.stored) {
          const int64_t row = (((int64_t)x.m_o * p.suffix_cap + j) * p.Hkv + hk) * 64;
          x.k_lo = *(const gu32x2*)(L.suffix_k + row + x.q8 * 4);
          x.k_hi = *(const gu32x2*)(L.suffix_k + row + 32 + x.q8 * 4);
          x.v = *(const gbf16x8*)(L.suffix_v + row + x.q8 * 8);
        }
      } else {
        x.m_o = b * p.R + min(x.f, p.R - 1);
        x.valid = x.f < p.R;
        fresh_slot = p.rows[x.m_o].kv_slot;
      }
      if (x.valid && !x.stored) {
        const gfloat* kp = gq + (int64_t)x.m_o * p.qkvd + p.qd + hk * 64 + x.q8 * 4;
        x.a = *(const gf32x4*)kp;
        x.bb = *(const gf32x4*)(kp + 32);
        const gfloat* cs = gcs + ((int64_t)x.m_o * 32 + x.q8 * 4) * 2;
        x.c0 = *(const gf32x4*)cs;
        x.c1 = *(const gf32x4*)(cs + 4);
        const gfloat* vp = gq + (int64_t)x.m_o * p.qkvd + p.qd + p.kvd + hk * 64 + x.q8 * 8;
        x.v0 = *(const gf32x4*)vp;
        x.v1 = *(const gf32x4*)(vp + 4);
      }
    }
  }

  // ---- Q operand: dims g4*8..+7 (k-step 0) and 32+g4*8..+7 (k-step 1) of this lane's query row, rotated, scaled
  const int tv = vq ? trunk_visible(rd, m, p.R) : 0;
  Bf8 qh[2], ql[2];
  {
    float a[8] = {qa0[0], qa0[1], qa0[2], qa0[3], qa1[0], qa1[1], qa1[2], qa1[3]};
    float bb[8] = {qb0[0], qb0[1], qb0[2], qb0[3], qb1[0], qb1[1], qb1[2], qb1[3]};
    float cc[16] = {qc0[0], qc0[1], qc0[2], qc0[3], qc1[0], qc1[1], qc1[2], qc1[3],
                    qc2[0], qc2[1], qc2[2], qc2[3], qc3[0], qc3[1], qc3[2], qc3[3]};
    const float scale = r_s[m] * 0.125f * kLog2e;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float c = cc[2 * i], sn = cc[2 * i + 1];
      float x0 = (a[i] * c - bb[i] * sn) * scale, x1 = (bb[i] * c + a[i] * sn) * scale;
      qh[0].u[i] = to_bf16(x0);
      qh[1].u[i] = to_bf16(x1);
      ql[0].u[i] = to_bf16(x0 - bf16_to_f32(qh[0].u[i]));
      ql[1].u[i] = to_bf16(x1 - bf16_to_f32(qh[1].u[i]));
    }
  }
  stamp(p, ph, 4);

  // ---- stage the fresh keys in LDS: K rows [64][72] (row padding against bank conflicts), V^T columns [64][72]
  bf16_t* kf_s = (bf16_t*)(lds + kFusedWaves * 4 * 64 + 64);
  bf16_t* vf_s = kf_s + 64 * 72;
  if (n_fb > 0) {
#pragma unroll
    for (int t = 0; t < 1; ++t) {
      Fresh& x = fr[t];
      if (threadIdx.x + t * kFusedThreads < nf8) {
        u32x2 k_lo = (u32x2){0u, 0u}, k_hi = (u32x2){0u, 0u};
        Bf8 vv;
        vv.w = (u32x4){0u, 0u, 0u, 0u};
        if (x.valid && x.stored) {
          k_lo = x.k_lo;
          k_hi = x.k_hi;
          vv.v = x.v;
        } else if (x.valid) {
          const float rs = r_s[x.m_o];
          float cc[8] = {x.c0[0], x.c0[1], x.c0[2], x.c0[3], x.c1[0], x.c1[1], x.c1[2], x.c1[3]};
          bf16_t x0[4], x1[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float c = cc[2 * e], sn = cc[2 * e + 1];
            x0[e] = to_bf16((x.a[e] * c - x.bb[e] * sn) * rs);
            x1[e] = to_bf16((x.bb[e] * c + x.a[e] * sn) * rs);
          }
          uint64_t p0 = pack_bf16x4(x0[0], x0[1], x0[2], x0[3]), p1 = pack_bf16x4(x1[0], x1[1], x1[2], x1[3]);
          k_lo = (u32x2){(uint32_t)p0, (uint32_t)(p0 >> 32)};
          k_hi = (u32x2){(uint32_t)p1, (uint32_t)(p1 >> 32)};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            vv.u[e] = to_bf16(x.v0[e] * rs);
            vv.u[4 + e] = to_bf16(x.v1[e] * rs);
          }
        }
        *(u32x2*)(kf_s + x.f * 72 + x.q8 * 4) = k_lo;
        *(u32x2*)(kf_s + x.f * 72 + 32 + x.q8 * 4) = k_hi;
#pragma unroll
        for (int e = 0; e < 8; ++e) vf_s[(x.q8 * 8 + e) * 72 + x.f] = vv.u[e];
      }
    }
    wg_barrier();
  }
  stamp(p, ph, 5);

  OnlineSoftmax st;
  st.m_run = -INFINITY;
  st.l_run = 0.f;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) st.acc[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // ---- stored trunk keys: RING blocks in flight.  Steady groups compute and reload unconditionally, the last group
  // only computes (blocks past the wavefront's last one are clamped duplicates with every key masked), so the load
  // counting stays exact and nothing is fetched twice.
  auto trunk_block = [&](const TrunkBlock& tb, int i) {
    const int kb = kb0 + (wave + kFusedWaves * i) * 32;
    f32x4 S[2];
    bool vis[8];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) S[tile] = score_tile<NPQ>(tb.k[tile][0], tb.k[tile][1], qh, ql);
#pragma unroll
    for (int e = 0; e < 8; ++e) vis[e] = i < n_mine && kb + g4 * 8 + e < tv;
    softmax_block<NPP>(st, S, vis, tb.vt);
  };
  int i0 = 0;
  for (; i0 + RING < n_mine; i0 += RING) {
#pragma unroll
    for (int r = 0; r < RING; ++r) {
      trunk_block(ring[r], i0 + r);
      load_trunk(ring[r], i0 + r + RING);
    }
  }
  if (n_mine > 0) {
#pragma unroll
    for (int r = 0; r < RING; ++r) trunk_block(ring[r], i0 + r);
  }
  stamp(p, ph, 6);
  // ---- fresh blocks continue the round-robin after the trunk blocks
  for (int blk = n_tb + ((wave - n_tb) & (kFusedWaves - 1)); blk < n_tb + n_fb; blk += kFusedWaves) {
    const int f0 = (blk - n_tb) * 32;
    f32x4 S[2];
    bool vis[8];
    bf16x8 vt[4];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      const bf16_t* kp = kf_s + (f0 + krow + tile * 4) * 72 + g4 * 8;
      S[tile] = score_tile<NPQ>(*(const bf16x8*)kp, *(const bf16x8*)(kp + 32), qh, ql);
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) vt[dt] = *(const bf16x8*)(vf_s + (dt * 16 + li) * 72 + f0 + g4 * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int f = f0 + g4 * 8 + e;
      vis[e] = vq && (is_branch ? ((f >> sl_log) == (li >> g_log) && (f & (p.SL - 1)) < p.suffix_len) : f <= rloc);
    }
    softmax_block<NPP>(st, S, vis, vt);
  }
  st.l_run = sum_over_rows(st.l_run);
  stamp(p, ph, 7);

  // the o-projection's operand planes: dims 4 dq .. 4 dq + 3 of query row qrow of this unit's tile
  auto write_att = [&](int qrow, int dq, f32x4 x4) {
    const int mm = b * p.R + qrow / p.G;
    const int k = (hk * p.G + qrow % p.G) * 64 + dq * 4;
    bf16_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      hi[i] = to_f16(x4[i]);
      lo[i] = to_f16(x4[i] - f16_to_f32(hi[i]));
    }
    const int64_t off = b_off<MT>(k, mm);
    st_u64(att_out + off, pack_bf16x4(hi[0], hi[1], hi[2], hi[3]));
    if (NPT == 2) st_u64(att_out + (int64_t)MP * p.qd + off, pack_bf16x4(lo[0], lo[1], lo[2], lo[3]));
  };
  // ---- the 8 wavefronts' partial softmaxes meet in LDS: acc [wave][dt][lane], (m, l) [wave][16]
  float* ml = (float*)(lds + kFusedWaves * 4 * 64);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) lds[(wave * 4 + dt) * 64 + lane] = st.acc[dt];
  if (g4 == 0) {
    ml[(wave * 16 + li) * 2] = st.m_run;
    ml[(wave * 16 + li) * 2 + 1] = st.l_run;
  }
  wg_barrier();
  if (threadIdx.x < 256) {
    const int q = threadIdx.x & 15, dq = threadIdx.x >> 4;       // query row of the tile, dims 4 dq .. 4 dq + 3
    float mmax = -INFINITY;
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) mmax = fmaxf(mmax, ml[(w * 16 + q) * 2]);
    const float m_use = mmax == -INFINITY ? 0.f : mmax;
    float lsum = 0.f;
    f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) {
      const float wgt = exp2_fast(ml[(w * 16 + q) * 2] - m_use);
      lsum += wgt * ml[(w * 16 + q) * 2 + 1];
      o += lds[(w * 4 + (dq >> 2)) * 64 + q + 16 * (dq & 3)] * wgt;
    }
    const int qrow = qt * 16 + q;
    if (qrow < RG) {
      if (p.NS == 1) {
        const float inv = 1.0f / lsum;
        write_att(qrow, dq, o * inv);
      } else {
        const int64_t pb = ((int64_t)(b * p.Hkv + hk) * p.NS + s) * (p.QT * 16) + qrow;
        if (dq == 0) st_u64(part_ml + pb * 2, pack_f32x2(mmax, lsum));
        st_f32x4(part_o + pb * 64 + dq * 4, o);
      }
    }
  }
  // ---- several key splits: this unit's arrival is counted once its partial softmax has left (write-through stores,
  // vmcnt 0); the count comes back while the fresh keys are appended below
  int* last_s = (int*)(vf_s + 64 * 72);
  if (SM && p.NS > 1) {
    __builtin_amdgcn_s_waitcnt(0);
    wg_barrier();
    if (threadIdx.x == 0) {
      unsigned* cnt = arrivals + (b * p.Hkv + hk) * p.QT + qt;
      const unsigned old = __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const int is_last = old + 1 == (unsigned)p.NS;
      if (is_last) __hip_atomic_store(cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next pass
      *last_s = is_last;
    }
  }
  // ---- append the keys and values computed in this pass for later passes, from their LDS copies: the row's private
  // suffix slot (branch) or its trunk position (extend).  Last, so that the stores are not in the way of any load.
  {
    const Fresh& x = fr[0];
    if (n_fb > 0 && (int)threadIdx.x < nf8 && x.valid && !x.stored) {
      const u32x2 k_lo = *(const u32x2*)(kf_s + x.f * 72 + x.q8 * 4), k_hi = *(const u32x2*)(kf_s + x.f * 72 + 32 + x.q8 * 4);
      Bf8 vv;
#pragma unroll
      for (int e = 0; e < 8; ++e) vv.u[e] = vf_s[(x.q8 * 8 + e) * 72 + x.f];
      if (is_branch) {
        const int64_t row = (((int64_t)x.m_o * p.suffix_cap + (p.suffix_len - 1)) * p.Hkv + hk) * 64;
        *(gu32x2*)(L.suffix_k + row + x.q8 * 4) = k_lo;
        *(gu32x2*)(L.suffix_k + row + 32 + x.q8 * 4) = k_hi;
        *(gbf16x8*)(L.suffix_v + row + x.q8 * 8) = vv.v;
      } else {
        const int64_t bb = PG ? ((int64_t)p.pages[(int64_t)b * p.page_stride + (fresh_slot >> 5)] * p.Hkv + hk) * 2048
                              : (int64_t)(b * p.Hkv + hk) * p.vt_stride * 64 + (int64_t)(fresh_slot >> 5) * 2048;
        const int64_t row = bb + (int64_t)(fresh_slot & 31) * 64;
        *(gu32x2*)(L.trunk_k + row + x.q8 * 4) = k_lo;
        *(gu32x2*)(L.trunk_k + row + 32 + x.q8 * 4) = k_hi;
        gbf16* vcol = (gbf16*)L.trunk_vt + bb + (x.q8 * 8) * 32 + (fresh_slot & 31);
#pragma unroll
        for (int e = 0; e < 8; ++e) vcol[e * 32] = vv.u[e];
      }
    }
  }
  // ---- the unit that arrived last of a tile's NS splits merges them, in split order whoever it is: no unit ever waits
  // for another, and the merge phase with its grid barrier is gone.  Its loads are agent-scope (coherent across the
  // XCDs); the other splits' stores were complete before their arrivals were counted.
  if (SM && p.NS > 1) {
    wg_barrier();
    if (*last_s != 0 && threadIdx.x < 256) {
      const int q = threadIdx.x & 15, dq = threadIdx.x >> 4;
      const int qrow = qt * 16 + q;
      if (qrow < RG) {
        constexpr int kMaxSplits = 16;
        const int64_t pb0 = ((int64_t)(b * p.Hkv + hk) * p.NS) * (p.QT * 16) + qrow, pstep = p.QT * 16;
        uint64_t mlv[kMaxSplits];
#pragma unroll
        for (int t = 0; t < kMaxSplits; ++t)
          mlv[t] = __hip_atomic_load((const uint64_t*)(part_ml + (pb0 + (t < p.NS ? t : 0) * pstep) * 2), __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
        float mmax = -INFINITY;
#pragma unroll
        for (int t = 0; t < kMaxSplits; ++t) mmax = t < p.NS ? fmaxf(mmax, __uint_as_float((unsigned)mlv[t])) : mmax;
        const float m_use = mmax == -INFINITY ? 0.f : mmax;
        float lsum = 0.f;
        f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t0 = 0; t0 < kMaxSplits; t0 += 4) {
          if (t0 < p.NS) {
            f32x4 ov[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) ov[t] = ld_f32x4_coherent(part_o + (pb0 + (t0 + t < p.NS ? t0 + t : 0) * pstep) * 64 + dq * 4);
#pragma unroll
            for (int t = 0; t < 4; ++t)
              if (t0 + t < p.NS) {
                const float wgt = exp2_fast(__uint_as_float((unsigned)mlv[t0 + t]) - m_use);
                lsum += wgt * __uint_as_float((unsigned)(mlv[t0 + t] >> 32));
                o += ov[t] * wgt;
              }
          }
        }
        write_att(qrow, dq, o * (1.0f / lsum));
      }
    }
  }
  wg_barrier();
  return true;
}

// The attention unit of the wide passes: NQ query tiles of one (sequence, KV head, key split) share every stored key
// and value block the unit pulls (a wide pass has 6 and more query tiles per sequence and head: units of one tile would
// pull the same trunk once per tile, and what bounds them is that pull, not their arithmetic).  Same method and same
// layouts as attn_unit; the qkv projections arrive with the norm's row scale applied.  Fresh keys: those of all the
// unit's query tiles (branch rows) or the pass's tokens (extend rows), staged once, NFI items per thread.
constexpr int kMultiFreshKeys = 192;   // LDS room: NQ x (rows per tile x slots per row) for NQ = 3, or the tokens of an extend
template <int MT, int MP, int NPQ, int NPP, int NQ, bool PG>
__device__ __forceinline__ void attn_unit_multi(const FusedParams& p, const FusedLayer& L, const float* qkv, int unit, f32x4* lds,
                                                bf16_t* att_out, float* part_o, float* part_ml, int ph) {
  const ThreadIds ids = fresh_thread_ids();
  const int lane = ids.lane, wave = ids.wave;
  const int li = lane & 15, g4 = lane >> 4;
  const int QG = (p.QT + NQ - 1) / NQ;        // groups of query tiles per (sequence, KV head)
  const int hk = unit % p.Hkv;
  int rem = unit / p.Hkv;
  const int qg = rem % QG;
  rem /= QG;
  const int s = rem % p.NS, b = rem / p.NS;
  const int g_log = 31 - __builtin_clz(p.G), sl_log = p.SL == 8 ? 3 : 4;   // G and SL are powers of two
  const int RG = p.R << g_log;
  const bool is_branch = p.is_branch != 0;
  const gfloat* gq = (const gfloat*)qkv;
  const gfloat* gcs = (const gfloat*)p.cos_sin;
  int qt[NQ], m[NQ], rloc[NQ];
  bool vq[NQ];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    qt[i] = qg * NQ + i;
    const int qr = qt[i] * 16 + li;
    vq[i] = qr < RG;
    const int qrc = vq[i] ? qr : RG - 1;
    rloc[i] = qrc >> g_log;
    m[i] = b * p.R + rloc[i];
  }

  // ---- issue: the first trunk blocks of this wavefront (block counts from the host's bound)
  const int kb0 = s * p.KPU;
  const int kend_ub = min(kb0 + p.KPU, p.tv_ub);
  const int n_tb = kend_ub > kb0 ? (kend_ub - kb0 + 31) >> 5 : 0;
  const int n_mine = n_tb > wave ? (n_tb - wave + kFusedWaves - 1) / kFusedWaves : 0;
  const int rpt = 16 >> g_log;                                // rows per query tile
  const int n_fresh_keys = is_branch ? (NQ * rpt) << sl_log : p.R;
  const int n_fb = s == 0 ? (n_fresh_keys + 31) >> 5 : 0;
  const int krow = (li >> 2) * 8 + (li & 3);                  // key of this lane's A-operand row in a block (tile 0)
  // PG (paged trunk, App. B "PagedAttention"): block j of sequence b is page p.pages[b][j] of a pool shared by all
  // sequences, a page = the same 4 KiB per head and operand as a block of the contiguous layouts.  Lane i of a wavefront
  // fetches the page of the wavefront's i-th block up front (one load), so the block loop itself stays free of
  // dependent loads; entries behind a sequence's allocation name page 0, which exists and holds zeros.
  const int64_t head0 = PG ? 0 : ((int64_t)(b * p.Hkv + hk) * p.vt_stride) * 64;
  const gbf16* kbase = (const gbf16*)L.trunk_k + head0 + g4 * 8;
  const gbf16* vbase = (const gbf16*)L.trunk_vt + head0 + li * 32 + g4 * 8;
  int pgs = 0;
  if constexpr (PG) pgs = p.pages[(int64_t)b * p.page_stride + min((kb0 >> 5) + wave + kFusedWaves * lane, p.page_stride - 1)];
  struct TrunkBlock {
    bf16x8 k[2][2];
    bf16x8 vt[4];
  };
  constexpr int RING = 2;
  TrunkBlock ring[RING];
  auto load_trunk = [&](TrunkBlock& tb, int i) {   // i-th block of this wavefront, clamped to its last one
    const int ic = max(min(i, n_mine - 1), 0);
    const int blk = wave + kFusedWaves * ic;
    const int kb = min(kb0 + blk * 32, p.vt_stride - 32);
    const int64_t bo = PG ? ((int64_t)__builtin_amdgcn_readlane(pgs, ic) * p.Hkv + hk) * 2048 : (int64_t)kb * 64;
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      const gbf16* kp = kbase + bo + (krow + tile * 4) * 64;
      tb.k[tile][0] = *(const gbf16x8*)kp;
      tb.k[tile][1] = *(const gbf16x8*)(kp + 32);
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) tb.vt[dt] = *(const gbf16x8*)(vbase + bo + dt * 16 * 32);
  };
#pragma unroll
  for (int i = 0; i < RING; ++i) load_trunk(ring[i], i);   // unconditional (a wavefront without blocks re-reads block 0)
  stamp(p, ph, 3);

  // ---- Q operands of the NQ tiles: dims g4*8..+7 (k-step 0) and 32+g4*8..+7 (k-step 1) of this lane's query rows,
  // rotated and scaled
  // (the loads of all NQ tiles go out before the first is used: one memory round trip instead of one per tile; the
  // scheduling barrier keeps the compiler from sinking them back next to their uses)
  int tv[NQ];
  Bf8 qh[NQ][2], ql[NQ][2];
  RowDesc rdv[NQ];
  f32x4 qraw[NQ][4], qcsv[NQ][4];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    rdv[i] = p.rows[m[i]];
    const int qrc = vq[i] ? qt[i] * 16 + li : RG - 1;
    const int hq = hk * p.G + (qrc & (p.G - 1));
    const gfloat* qp = gq + (int64_t)m[i] * p.qkvd + hq * 64 + g4 * 8;
    qraw[i][0] = *(const gf32x4*)qp;
    qraw[i][1] = *(const gf32x4*)(qp + 4);
    qraw[i][2] = *(const gf32x4*)(qp + 32);
    qraw[i][3] = *(const gf32x4*)(qp + 36);
    const gfloat* qcs = gcs + ((int64_t)m[i] * 32 + g4 * 8) * 2;
#pragma unroll
    for (int c4 = 0; c4 < 4; ++c4) qcsv[i][c4] = *(const gf32x4*)(qcs + 4 * c4);
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const RowDesc rd = rdv[i];
    const f32x4 qa0 = qraw[i][0], qa1 = qraw[i][1], qb0 = qraw[i][2], qb1 = qraw[i][3];
    const f32x4 qc0 = qcsv[i][0], qc1 = qcsv[i][1], qc2 = qcsv[i][2], qc3 = qcsv[i][3];
    tv[i] = vq[i] ? trunk_visible(rd, m[i], p.R) : 0;
    const float a[8] = {qa0[0], qa0[1], qa0[2], qa0[3], qa1[0], qa1[1], qa1[2], qa1[3]};
    const float bb[8] = {qb0[0], qb0[1], qb0[2], qb0[3], qb1[0], qb1[1], qb1[2], qb1[3]};
    const float cc[16] = {qc0[0], qc0[1], qc0[2], qc0[3], qc1[0], qc1[1], qc1[2], qc1[3],
                          qc2[0], qc2[1], qc2[2], qc2[3], qc3[0], qc3[1], qc3[2], qc3[3]};
    const float scale = 0.125f * kLog2e;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float c = cc[2 * e], sn = cc[2 * e + 1];
      const float x0 = (a[e] * c - bb[e] * sn) * scale, x1 = (bb[e] * c + a[e] * sn) * scale;
      qh[i][0].u[e] = to_bf16(x0);
      qh[i][1].u[e] = to_bf16(x1);
      ql[i][0].u[e] = to_bf16(x0 - bf16_to_f32(qh[i][0].u[e]));
      ql[i][1].u[e] = to_bf16(x1 - bf16_to_f32(qh[i][1].u[e]));
    }
  }

  stamp(p, ph, 4);
  // ---- stage the fresh keys in LDS: K rows [kMultiFreshKeys][72] (row padding against bank conflicts), V^T columns
  // [64][kMultiFreshKeys + 8]; item = (key f, rotary quad / 8-dim group q8), one after the other per thread
  constexpr int VS = kMultiFreshKeys + 8;
  bf16_t* kf_s = (bf16_t*)(lds + kFusedWaves * 4 * 64 + 64);
  bf16_t* vf_s = kf_s + kMultiFreshKeys * 72;
  const int nf8 = n_fb * 32 * 8;
  auto fresh_row = [&](int f, int& m_o, bool& valid, bool& stored) {
    if (is_branch) {
      const int rt = qg * NQ * rpt + (f >> sl_log), j = f & (p.SL - 1);
      m_o = b * p.R + min(rt, p.R - 1);
      valid = rt < p.R && j < p.suffix_len;
      stored = j < p.suffix_len - 1;
    } else {
      m_o = b * p.R + min(f, p.R - 1);
      valid = f < p.R;
      stored = false;
    }
  };
  if (n_fb > 0) {
    for (int it = threadIdx.x; it < nf8; it += kFusedThreads) {
      const int f = it >> 3, q8 = it & 7;
      int m_o;
      bool valid, stored;
      fresh_row(f, m_o, valid, stored);
      u32x2 k_lo = (u32x2){0u, 0u}, k_hi = (u32x2){0u, 0u};
      Bf8 vv;
      vv.w = (u32x4){0u, 0u, 0u, 0u};
      if (valid && stored) {
        const int64_t row = (((int64_t)m_o * p.suffix_cap + (f & (p.SL - 1))) * p.Hkv + hk) * 64;
        k_lo = *(const gu32x2*)(L.suffix_k + row + q8 * 4);
        k_hi = *(const gu32x2*)(L.suffix_k + row + 32 + q8 * 4);
        vv.v = *(const gbf16x8*)(L.suffix_v + row + q8 * 8);
      } else if (valid) {
        const gfloat* kp = gq + (int64_t)m_o * p.qkvd + p.qd + hk * 64 + q8 * 4;
        const f32x4 a = *(const gf32x4*)kp, bb = *(const gf32x4*)(kp + 32);
        const gfloat* cs = gcs + ((int64_t)m_o * 32 + q8 * 4) * 2;
        const f32x4 c0 = *(const gf32x4*)cs, c1 = *(const gf32x4*)(cs + 4);
        const gfloat* vp = gq + (int64_t)m_o * p.qkvd + p.qd + p.kvd + hk * 64 + q8 * 8;
        const f32x4 v0 = *(const gf32x4*)vp, v1 = *(const gf32x4*)(vp + 4);
        const float cc[8] = {c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
        bf16_t x0[4], x1[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float c = cc[2 * e], sn = cc[2 * e + 1];
          x0[e] = to_bf16(a[e] * c - bb[e] * sn);
          x1[e] = to_bf16(bb[e] * c + a[e] * sn);
        }
        const uint64_t p0 = pack_bf16x4(x0[0], x0[1], x0[2], x0[3]), p1 = pack_bf16x4(x1[0], x1[1], x1[2], x1[3]);
        k_lo = (u32x2){(uint32_t)p0, (uint32_t)(p0 >> 32)};
        k_hi = (u32x2){(uint32_t)p1, (uint32_t)(p1 >> 32)};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          vv.u[e] = to_bf16(v0[e]);
          vv.u[4 + e] = to_bf16(v1[e]);
        }
      }
      *(u32x2*)(kf_s + f * 72 + q8 * 4) = k_lo;
      *(u32x2*)(kf_s + f * 72 + 32 + q8 * 4) = k_hi;
#pragma unroll
      for (int e = 0; e < 8; ++e) vf_s[(q8 * 8 + e) * VS + f] = vv.u[e];
    }
    wg_barrier();
  }
  stamp(p, ph, 5);

  OnlineSoftmax st[NQ];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    st[i].m_run = -INFINITY;
    st[i].l_run = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) st[i].acc[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  // ---- stored trunk keys: RING blocks in flight, every block scored against all NQ query tiles
  auto trunk_block = [&](const TrunkBlock& tb, int i) {
    const int kb = kb0 + (wave + kFusedWaves * i) * 32;
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
      f32x4 S[2];
      bool vis[8];
#pragma unroll
      for (int tile = 0; tile < 2; ++tile) S[tile] = score_tile<NPQ>(tb.k[tile][0], tb.k[tile][1], qh[t], ql[t]);
#pragma unroll
      for (int e = 0; e < 8; ++e) vis[e] = i < n_mine && kb + g4 * 8 + e < tv[t];
      softmax_block<NPP>(st[t], S, vis, tb.vt);
    }
  };
  int i0 = 0;
  for (; i0 + RING < n_mine; i0 += RING) {
#pragma unroll
    for (int r = 0; r < RING; ++r) {
      trunk_block(ring[r], i0 + r);
      load_trunk(ring[r], i0 + r + RING);
    }
  }
  if (n_mine > 0) {
#pragma unroll
    for (int r = 0; r < RING; ++r) trunk_block(ring[r], i0 + r);
  }
  stamp(p, ph, 6);
  // ---- fresh blocks continue the round-robin after the trunk blocks
  for (int blk = n_tb + ((wave - n_tb) & (kFusedWaves - 1)); blk < n_tb + n_fb; blk += kFusedWaves) {
    const int f0 = (blk - n_tb) * 32;
    bf16x8 kk[2][2], vt[4];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      const bf16_t* kp = kf_s + (f0 + krow + tile * 4) * 72 + g4 * 8;
      kk[tile][0] = *(const bf16x8*)kp;
      kk[tile][1] = *(const bf16x8*)(kp + 32);
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) vt[dt] = *(const bf16x8*)(vf_s + (dt * 16 + li) * VS + f0 + g4 * 8);
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
      f32x4 S[2];
      bool vis[8];
#pragma unroll
      for (int tile = 0; tile < 2; ++tile) S[tile] = score_tile<NPQ>(kk[tile][0], kk[tile][1], qh[t], ql[t]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int f = f0 + g4 * 8 + e;
        vis[e] = vq[t] && (is_branch ? ((f >> sl_log) == t * rpt + (li >> g_log) && (f & (p.SL - 1)) < p.suffix_len) : f <= rloc[t]);
      }
      softmax_block<NPP>(st[t], S, vis, vt);
    }
  }

  stamp(p, ph, 7);
  // ---- the 8 wavefronts' partial softmaxes meet in LDS, one query tile after the other: acc [wave][dt][lane],
  // (m, l) [wave][16]
  float* ml = (float*)(lds + kFusedWaves * 4 * 64);
#pragma unroll
  for (int t = 0; t < NQ; ++t) {
    st[t].l_run = sum_over_rows(st[t].l_run);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) lds[(wave * 4 + dt) * 64 + lane] = st[t].acc[dt];
    if (g4 == 0) {
      ml[(wave * 16 + li) * 2] = st[t].m_run;
      ml[(wave * 16 + li) * 2 + 1] = st[t].l_run;
    }
    wg_barrier();
    if (threadIdx.x < 256) {
      const int q = threadIdx.x & 15, dq = threadIdx.x >> 4;       // query row of the tile, dims 4 dq .. 4 dq + 3
      float mmax = -INFINITY;
#pragma unroll
      for (int w = 0; w < kFusedWaves; ++w) mmax = fmaxf(mmax, ml[(w * 16 + q) * 2]);
      const float m_use = mmax == -INFINITY ? 0.f : mmax;
      float lsum = 0.f;
      f32x4 o = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < kFusedWaves; ++w) {
        const float wgt = exp2_fast(ml[(w * 16 + q) * 2] - m_use);
        lsum += wgt * ml[(w * 16 + q) * 2 + 1];
        o += lds[(w * 4 + (dq >> 2)) * 64 + q + 16 * (dq & 3)] * wgt;
      }
      const int qrow = (qg * NQ + t) * 16 + q;
      if (qrow < RG) {
        if (p.NS == 1) {
          const int mm = b * p.R + qrow / p.G;
          const int k = (hk * p.G + qrow % p.G) * 64 + dq * 4;
          const float inv = 1.0f / lsum;
          bf16_t hi[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) hi[e] = to_f16(o[e] * inv);      // (this unit serves wide passes only: fp16 activations)
          st_u64(att_out + b_off<MT>(k, mm), pack_bf16x4(hi[0], hi[1], hi[2], hi[3]));
        } else {
          const int64_t pb = ((int64_t)(b * p.Hkv + hk) * p.NS + s) * (p.QT * 16) + qrow;
          if (dq == 0) st_u64(part_ml + pb * 2, pack_f32x2(mmax, lsum));
          st_f32x4(part_o + pb * 64 + dq * 4, o);
        }
      }
    }
    wg_barrier();
  }
  stamp(p, ph, 1);
  // ---- append the keys and values computed in this pass for later passes, from their LDS copies: the row's private
  // suffix slot (branch) or its trunk position (extend)
  if (n_fb > 0) {
    for (int it = threadIdx.x; it < nf8; it += kFusedThreads) {
      const int f = it >> 3, q8 = it & 7;
      int m_o;
      bool valid, stored;
      fresh_row(f, m_o, valid, stored);
      if (!valid || stored) continue;
      const u32x2 k_lo = *(const u32x2*)(kf_s + f * 72 + q8 * 4), k_hi = *(const u32x2*)(kf_s + f * 72 + 32 + q8 * 4);
      Bf8 vv;
#pragma unroll
      for (int e = 0; e < 8; ++e) vv.u[e] = vf_s[(q8 * 8 + e) * VS + f];
      if (is_branch) {
        const int64_t row = (((int64_t)m_o * p.suffix_cap + (p.suffix_len - 1)) * p.Hkv + hk) * 64;
        *(gu32x2*)(L.suffix_k + row + q8 * 4) = k_lo;
        *(gu32x2*)(L.suffix_k + row + 32 + q8 * 4) = k_hi;
        *(gbf16x8*)(L.suffix_v + row + q8 * 8) = vv.v;
      } else {
        const int slot = p.rows[m_o].kv_slot;
        const int64_t bb = PG ? ((int64_t)p.pages[(int64_t)b * p.page_stride + (slot >> 5)] * p.Hkv + hk) * 2048
                              : (int64_t)(b * p.Hkv + hk) * p.vt_stride * 64 + (int64_t)(slot >> 5) * 2048;
        const int64_t row = bb + (int64_t)(slot & 31) * 64;
        *(gu32x2*)(L.trunk_k + row + q8 * 4) = k_lo;
        *(gu32x2*)(L.trunk_k + row + 32 + q8 * 4) = k_hi;
        gbf16* vcol = (gbf16*)L.trunk_vt + bb + (q8 * 8) * 32 + (slot & 31);
#pragma unroll
        for (int e = 0; e < 8; ++e) vcol[e * 32] = vv.u[e];
      }
    }
  }
  wg_barrier();
}

// Merge unit (only when the trunk is split over several units): one wavefront per (row, query head), lane = head
// dimension, merges the NS partial softmaxes and writes the attention output planes.
template <int MT, int MP, int NPT>
__device__ __forceinline__ void attn_merge_unit(const FusedParams& p, int unit, const float* part_o, const float* part_ml,
                                                bf16_t* att_out) {
  const int d = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int pair = unit * kFusedWaves + wave;
  if (pair >= p.M * p.Hq) return;
  const int m = pair / p.Hq, hq = pair - m * p.Hq;
  const int hk = hq / p.G, gq = hq - hk * p.G;
  const int b = m / p.R;
  const int qrow = (m - b * p.R) * p.G + gq;
  const int64_t pb0 = ((int64_t)(b * p.Hkv + hk) * p.NS) * (p.QT * 16) + qrow;
  const gfloat* gml = (const gfloat*)part_ml;
  const gfloat* go = (const gfloat*)part_o;
  float mmax = -INFINITY;
  for (int s = 0; s < p.NS; ++s) mmax = fmaxf(mmax, gml[(pb0 + (int64_t)s * (p.QT * 16)) * 2]);
  const float m_use = mmax == -INFINITY ? 0.f : mmax;
  float lsum = 0.f, o = 0.f;
  for (int s = 0; s < p.NS; ++s) {
    const int64_t pb = pb0 + (int64_t)s * (p.QT * 16);
    const float wgt = exp2_fast(gml[pb * 2] - m_use);
    lsum += wgt * gml[pb * 2 + 1];
    o += wgt * go[pb * 64 + d];
  }
  const float x = o / lsum;
  const bf16_t hi = to_f16(x);
  const bf16_t lo = to_f16(x - f16_to_f32(hi));
  // lanes d, d+1, d+2, d+3 -> one 8-byte store per plane from lane d (d % 4 == 0)
  uint32_t w = (uint32_t)hi | ((uint32_t)lo << 16);
  uint32_t w1 = __shfl_down(w, 1), w2 = __shfl_down(w, 2), w3 = __shfl_down(w, 3);
  if ((d & 3) == 0) {
    const int k = hq * 64 + d;
    const int64_t off = b_off<MT>(k, m);
    st_u64(att_out + off, pack_bf16x4((bf16_t)w, (bf16_t)w1, (bf16_t)w2, (bf16_t)w3));
    if (NPT == 2)
      st_u64(att_out + (int64_t)MP * p.qd + off,
             pack_bf16x4((bf16_t)(w >> 16), (bf16_t)(w1 >> 16), (bf16_t)(w2 >> 16), (bf16_t)(w3 >> 16)));
  }
}

// ---------------------------------------------------------------------------------------------- wide passes
// Passes of more than kFusedMaxRows rows (up to kFusedWideRows: the branch rows of a batch of sequences, App. C:
// B (K+1) F rows per step).  With hundreds of rows a linear layer is no longer a pure weight stream: every weight tile
// meets 24 row tiles, and what limits a compute unit is the rate at which it pulls operands from L2 (about 64 bytes
// per clock) and the latency of each pull, so the work of a layer is cut in two dimensions and every phase is a kernel
// of its own, shaped for its work (a wide step takes milliseconds: the dozens of launches cost little beside it).
//
// Linear layers (wide_gemm_kernel).  A "pair" = (4 feature tiles, one group of kWideGroup row tiles) over the whole
// reduction dimension.  A workgroup is 4 wavefronts, ONE per SIMD, so each may use all 512 vector registers: 96 hold
// the 24 accumulator tiles, the rest a ring of kWideRing register chunks, 7 of them (70 KiB per wavefront) in flight
// while one is multiplied: a compute unit has to keep about 200 KiB in flight to pull at L2 rate.  The wavefronts
// split the reduction dimension; each streams its own weight tiles (A operands, straight from the stream-order
// layout: two of its eight wavefront runs, and a k-slice of a K-split layer is just another piece of the range) and
// the matching activation tiles of the row group (B operands, one fp16 plane): 24 MFMAs per 10 KiB pulled.  The row
// groups of one set of feature tiles run on workgroups of ONE XCD (workgroup w runs on XCD w % 8), so the weights
// leave HBM once and the other row groups find them in that XCD's L2.  The four partial tiles meet in LDS (96 KiB) and
// are added in wavefront order.
constexpr int kWideTiles = kFusedWideRows / 16;
constexpr int kWideGroup = 6;
constexpr int kWideRing = 8;
constexpr int kWideThreads = 256, kWideWaves = 4;
constexpr int kWideQueryTiles = kFusedWideQueryTiles;   // query tiles that share a unit's pull of the stored keys

// plain stores the compiler does not count (see st_f32x4_uncounted)
__device__ __forceinline__ void st_u64_uncounted(void* p, uint64_t v) {
  asm volatile("global_store_dwordx2 %0, %1, off" : : "v"(p), "v"(v));
}
__device__ __forceinline__ void st_f32_uncounted(float* p, float v) {
  asm volatile("global_store_dword %0, %1, off" : : "v"(p), "v"(v));
}

// 1/rms of rows m_lo .. m_hi-1 of a wide pass into r_s[m] (LDS).  Wide passes keep the sums of squares of the residual
// stream per 64 features (the 4 feature tiles a workgroup of the producing kernel owns): ssq[feature quad][row].  All
// loads of a thread go out together (one memory round trip); 4 wavefronts; tmp: 4 x 64 floats of LDS.
template <int MP>
__device__ __forceinline__ void wide_row_scales(const FusedParams& p, const float* ssq, float* r_s, float* tmp, int m_lo, int m_hi) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_quads = p.d >> 6;
  const gfloat* src = (const gfloat*)ssq;
  for (int m0 = m_lo; m0 < m_hi; m0 += 128) {
    float sum[2] = {0.f, 0.f};
    for (int j0 = wave; j0 < n_quads; j0 += 4 * 8) {
      float v[2][8];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int m = m0 + 64 * h + lane;
        const int mc = m < m_hi ? m : m_hi - 1;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int j = j0 + 4 * i;
          v[h][i] = src[(int64_t)(j < n_quads ? j : j0) * MP + mc];
        }
      }
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 8; ++i) sum[h] += j0 + 4 * i < n_quads ? v[h][i] : 0.f;
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int m = m0 + 64 * h + lane;
      tmp[wave * 64 + lane] = sum[h];
      wg_barrier();
      if (wave == 0 && m < m_hi) r_s[m] = 1.0f / sqrtf((tmp[lane] + tmp[64 + lane] + tmp[128 + lane] + tmp[192 + lane]) / (float)p.d + p.eps);
      wg_barrier();
    }
  }
}

template <int MTG>
struct WideChunk {
  bf16x8 a[4];
  bf16x8 b[MTG];
};

struct WideEpi {
  float* out;          // QKV: [M][ld] projections with the norm's row scale applied; LOGITS: [M][ld] logits
  int64_t ld;
  const float* h_in;   // RESID
  float* h_out;
  const bf16_t* gain;
  bf16_t* xn_out;
  float* ssq_out;
  bf16_t* act_out;     // SWIGLU
  const float* ssq_in; // QKV, SWIGLU, LOGITS: per-feature-tile sums of squares of the input's residual stream
  int ph;              // phase id (for the optional clocks)
};

// ATW: feature tiles per unit of the layer's stream-order layout (2: qkv, o, down; 4: gate/up, LM head).
// D: chunks of the ring (kWideRing; half of it for reduction dimensions too short for whole turns of the full ring).
// MTG: row tiles per row group: kWideGroup, or half of it where that gives every workgroup of the grid a pair (the
// o- and down-projections have few feature tiles; smaller groups pull more bytes per MFMA but idle no compute unit).
template <int ATW, int EPI, int D, int MTG>
__global__ __launch_bounds__(kWideThreads) void wide_gemm_kernel(FusedParams p, FusedGemm g, const bf16_t* bsrc, WideEpi e) {
  constexpr int MP = kFusedWideRows, MTOT = kWideTiles, NT = 4 * MTG;
  extern __shared__ f32x4 red[];
  __shared__ float r_s[MP];
  __shared__ float ssq_s[NT * 16];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int KTW = g.KTW, KS = g.KS;
  const int NCH8 = KS * KTW;                        // k-tiles per pair in one of the layout's 8 wavefront runs
  const int NCH = 2 * NCH8;                         // k-tiles per pair of this wavefront (a multiple of D: host check)
  const int n_groups = g.n_units / KS;
  const int nq = ATW == 4 ? n_groups : n_groups >> 1;
  const int n_rg = (((p.M + 15) >> 4) + MTG - 1) / MTG;
  // the pairs of this workgroup: XCD x = blockIdx.x % 8 serves the tile sets q = x, x + 8, ..; its workgroups take
  // (set, row group) pairs t = wx, wx + per_xcd, .. with the row group running fastest
  const int x = (int)blockIdx.x & 7, wx = (int)blockIdx.x >> 3, per_xcd = (int)gridDim.x >> 3;
  const int nqx = x < nq ? (nq - x + 7) >> 3 : 0;
  const int tx = nqx * n_rg;
  const int n_my = wx < tx ? (tx - wx + per_xcd - 1) / per_xcd : 0;
  stamp(p, e.ph, 0);
  if (n_my == 0) return;

  f32x4 acc[4][MTG];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int t = 0; t < MTG; ++t) acc[j][t] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // The load cursor walks the chunks of this wavefront: pair after pair, in a pair the two wavefront runs of the
  // layout it covers, in a run the k-slices, in a slice KTW consecutive k-tiles.  Inside such a segment both operand
  // addresses advance by a constant; only a segment change (every KTW chunks) costs index arithmetic: scalar
  // divisions per chunk would take longer than the chunk's MFMAs.
  struct Cursor {
    const bf16_t* a;     // this wavefront's A tiles of the chunk (feature tile 0 of the set; ATW == 2: of its first unit)
    const bf16_t* b;     // B tile 0 of the row group at the chunk's k-tile
    int i, seg, n;       // k-tile in the segment, segment in the pair (run * KS + k-slice), pair ordinal
  };
  const int64_t a_step = (int64_t)ATW * 512;                     // next k-tile of a segment
  const int64_t a_unit2 = (int64_t)KS * kFusedWaves * KTW * 2 * 512;   // ATW == 2: from the set's first unit to its second
  const int64_t b_step = (int64_t)MTOT * 512;
  auto place = [&](Cursor& cu) {   // operand addresses at the start of segment cu.seg of pair cu.n (clamped to the last pair)
    const int t = wx + (cu.n < n_my ? cu.n : n_my - 1) * per_xcd;
    const int qh = t / n_rg;
    const int q = qh * 8 + x, rg = t - qh * n_rg;
    const int half = cu.seg >= KS ? 1 : 0;
    const int ks = cu.seg - half * KS;
    const int run = 2 * wave + half;                // which of the layout's 8 wavefront runs
    const int64_t unit = ATW == 4 ? (int64_t)q : (int64_t)(2 * q) * KS + ks;
    cu.a = g.w + ((unit * kFusedWaves + run) * KTW) * ATW * 512;
    cu.b = bsrc + ((int64_t)((ks * kFusedWaves + run) * KTW) * MTOT + rg * MTG) * 512;
  };
  auto advance = [&](Cursor& cu) {
    cu.a += a_step;
    cu.b += b_step;
    if (++cu.i == KTW) {
      cu.i = 0;
      if (++cu.seg == 2 * KS) { cu.seg = 0; ++cu.n; }
      place(cu);
    }
  };
  // (plain, cached loads also for the weights: the other row groups of the same feature tiles, on this XCD, find them
  // in its L2; a streaming hint would make every row group fetch them from memory again)
  auto load_chunk = [&](WideChunk<MTG>& ck, const Cursor& cu) {
    const gbf16x8* ap = (const gbf16x8*)cu.a + lane;
    if constexpr (ATW == 4) {
#pragma unroll
      for (int j = 0; j < 4; ++j) ck.a[j] = ap[j * 64];
    } else {
      const gbf16x8* ap2 = (const gbf16x8*)(cu.a + a_unit2) + lane;
      ck.a[0] = ap[0];
      ck.a[1] = ap[64];
      ck.a[2] = ap2[0];
      ck.a[3] = ap2[64];
    }
    const gbf16x8* bp = (const gbf16x8*)cu.b + lane;
#pragma unroll
    for (int t = 0; t < MTG; ++t) ck.b[t] = bp[t * 64];
  };
  auto mfma_chunk = [&](const WideChunk<MTG>& ck) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int t = 0; t < MTG; ++t) acc[j][t] = mfma16_f16(ck.a[j], ck.b[t], acc[j][t]);
  };

  // 1/rms of the rows this workgroup's pairs cover: one row group if per_xcd is a multiple of n_rg, else all rows
  // (before the ring's loads, which fill the load counter)
  if (EPI != FE_RESID) {
    const bool one_group = per_xcd % n_rg == 0;
    const int m_lo = one_group ? (wx % n_rg) * MTG * 16 : 0;
    wide_row_scales<MP>(p, e.ssq_in, r_s, (float*)red, m_lo, min(p.M, one_group ? m_lo + MTG * 16 : p.M));
  }

  WideChunk<MTG> ring[D];
  Cursor cu{nullptr, nullptr, 0, 0, 0};
  place(cu);
#pragma unroll
  for (int s = 0; s < D - 1; ++s) { load_chunk(ring[s], cu); advance(cu); }
  stamp(p, e.ph, 1);

  stamp(p, e.ph, 3);
  for (int n = 0; n < n_my; ++n) {
    const int t = wx + n * per_xcd;
    const int q = (t / n_rg) * 8 + x, rg = t - (t / n_rg) * n_rg;
    for (int c = 0; c < NCH; c += D) {
#pragma unroll
      for (int s = 0; s < D; ++s) {
        load_chunk(ring[(s + D - 1) % D], cu);
        advance(cu);
        mfma_chunk(ring[s]);
      }
    }
    if (n == 0) stamp(p, e.ph, 4);
    // ---- end of a pair: the 4 wavefronts' partial tiles meet in LDS; every wavefront sums its 6 of the 24 tiles in
    // wavefront order and runs their epilogue
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int tt = 0; tt < MTG; ++tt) {
        red[(wave * NT + j * MTG + tt) * 64 + lane] = acc[j][tt];
        acc[j][tt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
    wg_barrier();
    auto total = [&](int idx) {
      f32x4 v = red[idx * 64 + lane];
#pragma unroll
      for (int w = 1; w < kWideWaves; ++w) v += red[(w * NT + idx) * 64 + lane];
      return v;
    };
    const int f4 = (lane >> 4) * 4;
    if constexpr (EPI == FE_SWIGLU) {
      // feature tiles 0, 1 of the set are gate, 2, 3 the matching up tiles
      for (int idx = wave; idx < 2 * MTG; idx += kWideWaves) {
        const int j = idx / MTG, tt = idx - j * MTG;
        const f32x4 gv = total(idx), uv = total(idx + 2 * MTG);
        const int m = (rg * MTG + tt) * 16 + (lane & 15);
        if (m < p.M) {
          const float rs = r_s[m];
          bf16_t hi[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float gg = gv[i] * rs, uu = uv[i] * rs;
            hi[i] = to_f16(gg / (1.0f + __expf(-gg)) * uu);
          }
          const int k = q * 32 + j * 16 + f4;      // input index of the down-projection
          st_u64_uncounted(e.act_out + b_off<MTOT>(k, m), pack_bf16x4(hi[0], hi[1], hi[2], hi[3]));
        }
      }
    } else {
      for (int idx = wave; idx < NT; idx += kWideWaves) {
        const int j = idx / MTG, tt = idx - j * MTG;
        const f32x4 v = total(idx);
        const int m = (rg * MTG + tt) * 16 + (lane & 15);
        const int tile = q * 4 + j;
        const int nn = tile * 16 + f4;
        if (tile >= g.NT) continue;
        if constexpr (EPI == FE_QKV || EPI == FE_LOGITS) {
          if (m < p.M) st_f32x4_uncounted(e.out + (int64_t)m * e.ld + nn, v * r_s[m]);
        } else {
          // residual stream: new h, (h * gain) as one fp16 plane for the next linear layer, this tile's sum of squares
          f32x4 hn = v;
          float ss = 0.f;
          if (m < p.M) {
            hn += *(const gf32x4*)(e.h_in + (int64_t)m * p.d + nn);
            const u32x2 gb = *(const gu32x2*)(e.gain + nn);
            st_f32x4_uncounted(e.h_out + (int64_t)m * p.d + nn, hn);
            const float gg[4] = {__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xffff0000u), __uint_as_float(gb.y << 16),
                                 __uint_as_float(gb.y & 0xffff0000u)};
            bf16_t hi[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              hi[i] = to_f16(hn[i] * gg[i]);
              ss += hn[i] * hn[i];
            }
            st_u64_uncounted(e.xn_out + b_off<MTOT>(nn, m), pack_bf16x4(hi[0], hi[1], hi[2], hi[3]));
          }
          ss += __shfl_xor(ss, 16);
          ss += __shfl_xor(ss, 32);
          if (lane < 16) ssq_s[idx * 16 + lane] = ss;     // this feature tile's sum of squares per row
        }
      }
    }
    wg_barrier();
    if constexpr (EPI == FE_RESID) {
      // the set's 4 feature tiles, added in tile order: one sum per (64 features, row)
      const int tt = (int)threadIdx.x >> 4, r = (int)threadIdx.x & 15;
      const int m = (rg * MTG + tt) * 16 + r;
      if (tt < MTG && m < p.M && q * 4 < g.NT) {
        float ss = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) ss += q * 4 + j < g.NT ? ssq_s[(j * MTG + tt) * 16 + r] : 0.f;
        st_f32_uncounted(e.ssq_out + q * MP + m, ss);
      }
      wg_barrier();
    }
    if (n == 0) stamp(p, e.ph, 5);
  }
  stamp(p, e.ph, 2);
}

// The two large linear layers of a wide pass (gate/up + SwiGLU, LM head; stream-order units of 4 feature tiles, no
// K-split).  Here the feature dimension is long enough to give every workgroup 16 feature tiles: the 4 wavefronts take
// one unit each over the WHOLE reduction dimension (a unit's weight tiles are one contiguous run of memory), and the
// activation tiles of the row group, which all four need, come through LDS: staged 8 k-tiles (48 KiB) at a time, double
// buffered, one workgroup barrier per stage.  Per k-tile a workgroup pulls 16 KiB of weights and 6 KiB of activations
// for 96 MFMAs (the split-K kernel above: 40 KiB), and nothing has to be reduced across wavefronts: the epilogue runs
// from the accumulators.  Weights ride a ring of 8 register chunks that is refilled one stage ahead.
// The MFMAs are 32x32x16: a wavefront that has its SIMD to itself issues one 16x16x32 per 28 clocks (measured: 1.44 of
// 2.5 PFLOP/s over the chip) but 32x32x16, twice the work per instruction, back to back (2.23).  Both operands stay in
// their 16x16x32 tile order in memory and LDS: a 32x32x16 operand is the k-half h of two neighbouring tiles, and lane l
// takes its 16 bytes from lane (l & 15) + 16 (l >> 5) + 32 h of tile (l >> 4) & 1, a fixed offset per lane.
constexpr int kWideStage = 8;   // k-tiles per LDS stage of the activation operand

template <int EPI>
__global__ __launch_bounds__(kWideThreads) void wide_gemm_lds_kernel(FusedParams p, FusedGemm g, const bf16_t* bsrc, WideEpi e) {
  constexpr int MP = kFusedWideRows, MTOT = kWideTiles, MTG = kWideGroup, KC = kWideStage;
  constexpr int STAGE = KC * MTG * 64;               // 16-byte vectors per stage
  constexpr int BL = STAGE / kWideThreads;           // staging loads per thread and stage (12)
  extern __shared__ f32x4 lds[];                     // [2][KC][MTG][64] B-operand vectors
  __shared__ float r_s[MP];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int NKT = g.KTW * kFusedWaves;               // k-tiles of the reduction dimension
  const int NST = NKT / KC;                          // stages per pair
  const int n_sets = (g.n_units + 3) >> 2;
  const int n_rg = (((p.M + 15) >> 4) + MTG - 1) / MTG;
  const int x = (int)blockIdx.x & 7, wx = (int)blockIdx.x >> 3, per_xcd = (int)gridDim.x >> 3;
  const int nqx = x < n_sets ? (n_sets - x + 7) >> 3 : 0;
  const int tx = nqx * n_rg;
  const int n_my = wx < tx ? (tx - wx + per_xcd - 1) / per_xcd : 0;
  stamp(p, e.ph, 0);
  if (n_my == 0) return;

  // ---- 1/rms of the rows this workgroup's pairs cover (one row group if per_xcd is a multiple of n_rg, else all rows)
  {
    const bool one_group = per_xcd % n_rg == 0;
    const int m_lo = one_group ? (wx % n_rg) * MTG * 16 : 0;
    wide_row_scales<MP>(p, e.ssq_in, r_s, (float*)lds, m_lo, min(p.M, one_group ? m_lo + MTG * 16 : p.M));
  }
  stamp(p, e.ph, 1);

  constexpr int MT32 = MTG / 2;                      // 32-row tiles of a row group
  static_assert(MTG % 2 == 0, "row tiles pair up into 32-row MFMA operands");
  const int lsrc = ((lane >> 4) & 1) * 64 + (lane & 15) + ((lane >> 5) << 4);   // operand vector of this lane (k-half 0)
  auto zero_acc = [](f32x16& a) {
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = 0.f;
  };
  f32x16 acc[2][MT32];                               // [32 features: tiles 0-1 / 2-3 of the unit][32 rows]
#pragma unroll
  for (int f = 0; f < 2; ++f)
#pragma unroll
    for (int t = 0; t < MT32; ++t) zero_acc(acc[f][t]);

  auto pair_of = [&](int n, int& set, int& rg) {
    const int t = wx + (n < n_my ? n : n_my - 1) * per_xcd;
    const int qh = t / n_rg;
    set = qh * 8 + x;
    rg = t - qh * n_rg;
  };
  // this thread's BL vectors of a stage: vector v = tid + 256 i of [KC][MTG][64] sits at k-tile v / (MTG 64), row tile
  // (v / 64) % MTG, lane v % 64 of the activation matrix [k-tile][MTOT][64]
  int64_t b_rel[BL];
#pragma unroll
  for (int i = 0; i < BL; ++i) {
    const int v = (int)threadIdx.x + kWideThreads * i;
    const int kt = v / (MTG * 64), r2 = v - kt * (MTG * 64);
    b_rel[i] = ((int64_t)kt * MTOT * 64 + r2) * 8;
  }
  struct Cursor { int n, s; const bf16_t* a; const bf16_t* b; };   // pair ordinal, stage; operand addresses of that stage
  auto place = [&](Cursor& cu) {
    int set, rg;
    pair_of(cu.n, set, rg);
    const int unit = min(set * 4 + wave, g.n_units - 1);
    cu.a = g.w + ((int64_t)unit * NKT + cu.s * KC) * 4 * 512;
    cu.b = bsrc + ((int64_t)(cu.s * KC) * MTOT + rg * MTG) * 512;
  };
  auto next_stage = [&](Cursor& cu) {
    if (++cu.s == NST) { cu.s = 0; ++cu.n; }
    place(cu);
  };
  bf16x8 ring[KC][4];
  bf16x8 breg[BL];
  auto load_b = [&](const Cursor& cu) {
#pragma unroll
    for (int i = 0; i < BL; ++i) breg[i] = *(const gbf16x8*)(cu.b + b_rel[i]);
  };
  auto store_b = [&](int buf) {
#pragma unroll
    for (int i = 0; i < BL; ++i) *(bf16x8*)&lds[buf * STAGE + (int)threadIdx.x + kWideThreads * i] = breg[i];
  };
  auto load_a = [&](const Cursor& cu, int j) {       // ring[j][2 f + h]: features 32 f .. 32 f + 31 of the unit, k-half h
    const gbf16x8* ap = (const gbf16x8*)(cu.a + (int64_t)j * 4 * 512) + lsrc;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) ring[j][jj] = ap[(jj >> 1) * 128 + (jj & 1) * 32];
  };

  // ---- prologue: stage 0 of the first pair
  Cursor cu{0, 0, nullptr, nullptr};
  place(cu);
  load_b(cu);
  // the ring is requested in the order the loop refills it: the wait for chunk j inside the loop is computed from BOTH
  // ways into the loop, and a prologue that had requested chunk 0 last would make every stage wait for the whole ring
#pragma unroll
  for (int j = 0; j < KC; ++j) {
    __builtin_amdgcn_sched_barrier(0);
    load_a(cu, j);
  }
  __builtin_amdgcn_sched_barrier(0);
  store_b(0);
  wg_barrier();
  stamp(p, e.ph, 3);

  int buf = 0;
  for (int n = 0; n < n_my; ++n) {
    int set, rg;
    pair_of(n, set, rg);
    for (int st = 0; st < NST; ++st) {
      next_stage(cu);                                // the stage after this one (clamped past the end: loaded, never used)
      load_b(cu);
      __builtin_amdgcn_sched_barrier(0);
      const bf16x8* bs = (const bf16x8*)&lds[buf * STAGE] + lsrc;
      // the activation tiles of k-tile j + 1 leave LDS while the MFMAs of k-tile j run: one wavefront per SIMD has no
      // neighbour to hide an LDS round trip behind.  bt[..][2 t + h]: rows 32 t .. 32 t + 31 of the group, k-half h
      bf16x8 bt[2][MTG];
#pragma unroll
      for (int t = 0; t < MTG; ++t) bt[0][t] = bs[(t >> 1) * 128 + (t & 1) * 32];
#pragma unroll
      for (int j = 0; j < KC; ++j) {
        if (j + 1 < KC) {
#pragma unroll
          for (int t = 0; t < MTG; ++t) bt[(j + 1) & 1][t] = bs[((j + 1) * MTG + (t >> 1) * 2) * 64 + (t & 1) * 32];
        }
        // (pinned in front of the MFMAs: the scheduler otherwise issues these reads behind them, into the registers the
        // MFMAs have just released, and every k-tile starts with an LDS round trip)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int t = 0; t < MT32; ++t)
              acc[f][t] = mfma32_f16(ring[j][2 * f + h], bt[j & 1][2 * t + h], acc[f][t]);
        load_a(cu, j);
        // the refill stays here, a whole stage ahead of its use: left alone, the instruction scheduler sinks it to just
        // before that use to save registers, and every k-tile then waits a full memory latency
        __builtin_amdgcn_sched_barrier(0);
      }
      store_b(buf ^ 1);
      wg_barrier();
      buf ^= 1;
    }
    if (n == 0) stamp(p, e.ph, 4);
    // ---- epilogue straight from the accumulators: this wavefront's unit (4 feature tiles) x the row group.  Registers
    // 4 q .. 4 q + 3 of a 32x32 accumulator: features 8 q + 4 (lane >> 5) .. + 3 of the 32, row lane & 31
    const int unit = set * 4 + wave;
    const int f4 = (lane >> 5) * 4;
    if (unit < g.n_units) {
#pragma unroll
      for (int t = 0; t < MT32; ++t) {
        const int m = (rg * MTG + 2 * t) * 16 + (lane & 31);
        if (m < p.M) {
          const float rs = r_s[m];
          if constexpr (EPI == FE_SWIGLU) {
            // feature tiles 0, 1 of the unit are gate, 2, 3 the matching up tiles
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              bf16_t hi[4];
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                const float gg = acc[0][t][4 * q + i] * rs, uu = acc[1][t][4 * q + i] * rs;
                hi[i] = to_f16(gg / (1.0f + __expf(-gg)) * uu);
              }
              const int k = unit * 32 + 8 * q + f4;       // input index of the down-projection
              st_u64_uncounted(e.act_out + b_off<MTOT>(k, m), pack_bf16x4(hi[0], hi[1], hi[2], hi[3]));
            }
          } else {
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int n0 = unit * 64 + f * 32 + 8 * q + f4;
                const f32x4 v = (f32x4){acc[f][t][4 * q], acc[f][t][4 * q + 1], acc[f][t][4 * q + 2], acc[f][t][4 * q + 3]};
                if ((n0 >> 4) < g.NT) st_f32x4_uncounted(e.out + (int64_t)m * e.ld + n0, v * rs);
              }
          }
        }
      }
    }
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int t = 0; t < MT32; ++t) zero_acc(acc[f][t]);
    if (n == 0) stamp(p, e.ph, 5);
  }
  stamp(p, e.ph, 2);
}

// The other phases of a wide pass (embedding, attention, merge of key splits, final hidden states), one launch each:
// the narrow pass's units over a workspace of kFusedWideRows rows, one fp16 plane per tensor.
template <class PL, bool PG>
__global__ __launch_bounds__(kFusedThreads) void wide_kernel(FusedParams p, int ph) {
  constexpr int MP = kFusedWideRows, MTOT = kWideTiles;
  extern __shared__ f32x4 red[];
  __shared__ float r_s[MP];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t h_stride = (int64_t)MP * p.d;
  const int64_t ssq_stride = (int64_t)(p.d >> 4) * MP;
  const int lm_phase = fused_last_phase(p.L);
  const int l = ph == 0 ? 0 : (ph == lm_phase ? p.L - 1 : (ph - 1) / 6);
  const int sub = ph == 0 ? -1 : (ph == lm_phase ? 6 : (ph - 1) % 6);
  const FusedLayer L = p.layers[l];
  float* qkv = p.qkv + (int64_t)l * MP * p.qkvd;
  bf16_t* att = p.att + (int64_t)l * 2 * MP * p.qd;
  float* part_o = p.part_o + (int64_t)l * p.part_layer_stride * 64;
  float* part_ml = p.part_ml + (int64_t)l * p.part_layer_stride * 2;
  stamp(p, ph, 0);
  if (sub == -1) {
    // embedding gather: residual stream version 0, (h * gain) as one fp16 plane, sums of squares per 64 features
    for (int u = blockIdx.x; u < (p.d >> 6); u += gridDim.x) {
      for (int t = wave; t < ((p.M + 15) >> 4); t += kFusedWaves) {
        const int m = t * 16 + (lane & 15);
        int tok = p.tokens[min(m, p.M - 1)];
        tok = tok < 0 ? 0 : (tok >= p.V ? p.V - 1 : tok);
        float ss = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int n = (u * 4 + j) * 16 + (lane >> 4) * 4;
          const u32x2 eb = *(const gu32x2*)(p.embed + (int64_t)tok * p.d + n);
          const u32x2 gb = *(const gu32x2*)(L.attn_norm + n);
          const float hv[4] = {__uint_as_float(eb.x << 16), __uint_as_float(eb.x & 0xffff0000u), __uint_as_float(eb.y << 16),
                               __uint_as_float(eb.y & 0xffff0000u)};
          const float gg[4] = {__uint_as_float(gb.x << 16), __uint_as_float(gb.x & 0xffff0000u), __uint_as_float(gb.y << 16),
                               __uint_as_float(gb.y & 0xffff0000u)};
          if (m < p.M) {
            *(gf32x4*)(p.h + (int64_t)m * p.d + n) = (f32x4){hv[0], hv[1], hv[2], hv[3]};
            bf16_t hi[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              hi[i] = to_f16(hv[i] * gg[i]);
              ss += hv[i] * hv[i];
            }
            *(uint64_t*)(p.xn + b_off<MTOT>(n, m)) = pack_bf16x4(hi[0], hi[1], hi[2], hi[3]);
          }
        }
        ss += __shfl_xor(ss, 16);
        ss += __shfl_xor(ss, 32);
        if (m < p.M && lane < 16) p.ssq[(int64_t)u * MP + m] = ss;
      }
    }
  } else if (sub == 1) {
    for (int u = blockIdx.x; u < p.n_attn_units; u += gridDim.x)
      attn_unit_multi<MTOT, MP, PL::q, PL::p, kWideQueryTiles, PG>(p, L, qkv, u, red, att, part_o, part_ml, ph);
  } else if (sub == 2) {
    for (int u = blockIdx.x; u < p.n_pair_units; u += gridDim.x) attn_merge_unit<MTOT, MP, 1>(p, u, part_o, part_ml, att);
  } else if (sub == 6 && p.hidden) {
    // final-norm hidden states: workgroup per row, the row's scale from the tile sums
    const int v = 2 * p.L;
    const gfloat* hv = (const gfloat*)(p.h + (int64_t)v * h_stride);
    const gfloat* sq = (const gfloat*)(p.ssq + (int64_t)v * ssq_stride);
    float* tmp = (float*)red;
    for (int m = blockIdx.x; m < p.M; m += gridDim.x) {
      float s = 0.f;
      for (int j = threadIdx.x; j < (p.d >> 6); j += kFusedThreads) s += sq[(int64_t)j * MP + m];
      for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
      if (lane == 0) tmp[wave] = s;
      wg_barrier();
      float tot = 0.f;
      for (int w = 0; w < kFusedWaves; ++w) tot += tmp[w];
      const float rs = 1.0f / sqrtf(tot / (float)p.d + p.eps);
      for (int c = threadIdx.x; c < p.d; c += kFusedThreads)
        p.hidden[(int64_t)m * p.hidden_ld + c] = hv[(int64_t)m * p.d + c] * bf16_to_f32(p.final_norm[c]) * rs;
      wg_barrier();
    }
  }
  stamp(p, ph, 2);
}

// ---------------------------------------------------------------------------------------------- the kernel
// Register chunks in flight per wavefront.  DEEP needs the k-tiles per wavefront of every linear layer to be a
// multiple of 8 (one feature tile per unit) / 4 (four per unit); the shallow set needs multiples of 2.
template <int MT, bool DEEP, int NP> struct Depth {
  static constexpr int a4 = !DEEP ? 2 : (MT * NP > 4 ? 2 : 4);   // four feature tiles per unit
};

template <int MT, bool DEEP, class PL, bool PG, bool SM>
__global__ __launch_bounds__(kFusedThreads) void fused_kernel(FusedParams p, int first, int last, int persistent) {
  constexpr int MP = kFusedMaxRows;
  extern __shared__ f32x4 red[];
  __shared__ float r_s[64];
  __shared__ int dead;
  if (threadIdx.x == 0) dead = 0;
  wg_barrier();
  // The barrier counts on from where the previous launch stopped (its last epoch is kept in a word of its own), so
  // the barrier words never have to be cleared between launches.
  Grid grid{p.bar, p.err, persistent ? p.bar[kBarEpochWord] : 0u, persistent, p.nwg, &dead, p.spin_limit};
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t h_stride = (int64_t)MP * p.d;
  const int64_t ssq_stride = (int64_t)(p.d >> 4) * MP;
  const int lm_phase = fused_last_phase(p.L);

  for (int ph = first; ph <= last; ++ph) {
    // the merge phase: none with one key split, and none where the attention units merge their splits themselves
    if ((SM || p.NS == 1) && ph > 0 && ph < lm_phase && (ph - 1) % 6 == 2) continue;
    const int l = ph == 0 ? 0 : (ph == lm_phase ? p.L - 1 : (ph - 1) / 6);
    const int sub = ph == 0 ? -1 : (ph == lm_phase ? 6 : (ph - 1) % 6);
    // group sync (see group_wait): no grid barrier between a layer's qkv phase and its attention phase
    const bool gs = persistent && p.qkv_ug > 0;
    const bool do_wait = persistent && ph > first && !(gs && sub == 1);
    stamp(p, ph, 0);
    if (ph == 0 && p.prof && threadIdx.x == 0) {
      unsigned xcc;
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
      p.prof[(int64_t)7 * p.nwg + blockIdx.x] = xcc;   // phase 0, slot 7: the XCD this workgroup runs on
    }
    const FusedLayer L = p.layers[l];
    float* qkv = p.qkv + (int64_t)l * MP * p.qkvd;
    bf16_t* att = p.att + (int64_t)l * 2 * MP * p.qd;
    bf16_t* act = p.act + (int64_t)l * 2 * MP * p.ffn;

    // ---- what a linear-layer phase streams, reads and writes
    FusedGemm g{};
    const bf16_t* bsrc = nullptr;
    int64_t bplane = 0;
    int epi = 0;
    EpiArgs e{};
    const float* ssq_in = nullptr;
    // the unit of this workgroup in the phases of at most one unit per workgroup: the workgroup's index, or, with group
    // sync, the qkv units of KV head gq's group (2 G for its query heads, 2 for its keys, 2 for its values, 32
    // features each) on workgroups 7 - gq, 15 - gq, ..: the XCD on which that head's attention units run
    int my_unit = (int)blockIdx.x;
    int qkv_flag = -1;    // word of the flags this workgroup sets after its qkv unit
    if (gs && sub == 0) {
      const int gq = 7 - ((int)blockIdx.x & 7), jj = (int)blockIdx.x >> 3;
      my_unit = -1;
      if (gq < p.Hkv && jj < p.qkv_ug) {
        const int nq = 2 * p.G;
        my_unit = jj < nq ? gq * nq + jj : (jj < nq + 2 ? 2 * p.Hq + 2 * gq + (jj - nq) : 2 * p.Hq + 2 * p.Hkv + 2 * gq + (jj - nq - 2));
        qkv_flag = (l * 8 + gq) * 16 + jj;
      }
    }
    // K-split scratch of this phase instance (sub 0, 3, 5 -> slot 0, 1, 2)
    const int fix_slot = l * 3 + (sub == 0 ? 0 : (sub == 3 ? 1 : 2));
    e.fix_buf = p.fix_buf + (int64_t)fix_slot * p.fix_stride;
    if (sub == 0) {
      g = L.qkv; bsrc = p.xn + (int64_t)(2 * l) * 2 * h_stride; bplane = h_stride; epi = FE_QKV;
      e.out = qkv; e.ld = p.qkvd;
      // the attention phase finds this layer's row scales in LDS; attention units are dealt out from the far end of
      // the grid, so (few rows) the workgroups that compute them here are not the ones that hold a qkv unit
      if (p.nwg - 1 - (int)blockIdx.x < p.n_attn_units) ssq_in = p.ssq + (int64_t)(2 * l) * ssq_stride;
    } else if (sub == 3 || sub == 5) {
      const int v = sub == 3 ? 2 * l + 1 : 2 * l + 2;
      g = sub == 3 ? L.o : L.down;
      bsrc = sub == 3 ? att : act;
      bplane = sub == 3 ? (int64_t)MP * p.qd : (int64_t)MP * p.ffn;
      epi = FE_RESID;
      e.h_in = p.h + (int64_t)(v - 1) * h_stride;
      e.h_out = p.h + (int64_t)v * h_stride;
      e.gain = sub == 3 ? L.mlp_norm : (l + 1 < p.L ? p.layers[l + 1].attn_norm : p.final_norm);
      e.xn_out = p.xn + (int64_t)v * 2 * h_stride;
      e.ssq_out = p.ssq + (int64_t)v * ssq_stride;
    } else if (sub == 4) {
      const int v = 2 * l + 1;
      g = L.gu; bsrc = p.xn + (int64_t)v * 2 * h_stride; bplane = h_stride; epi = FE_SWIGLU;
      e.act_out = act;
      ssq_in = p.ssq + (int64_t)v * ssq_stride;
    } else if (sub == 6) {
      const int v = 2 * p.L;
      g = p.lm; bsrc = p.xn + (int64_t)v * 2 * h_stride; bplane = h_stride; epi = FE_LOGITS;
      e.out = p.logits; e.ld = p.logits_ld;
      ssq_in = p.ssq + (int64_t)v * ssq_stride;
      if (!p.logits) g.n_units = 0;   // hidden states only
    }

    if (sub == -1) {
      // ---- embedding gather: residual stream version 0
      for (int u = blockIdx.x; u < (p.d >> 4); u += p.nwg) {
        if (wave < MT) {
          const int m = wave * 16 + (lane & 15);
          const int n = u * 16 + (lane >> 4) * 4;
          int tok = p.tokens[min(m, p.M - 1)];
          tok = tok < 0 ? 0 : (tok >= p.V ? p.V - 1 : tok);
          u32x2 eb = *(const gu32x2*)(p.embed + (int64_t)tok * p.d + n);
          f32x4 hn = (f32x4){__uint_as_float(eb.x << 16), __uint_as_float(eb.x & 0xffff0000u),
                             __uint_as_float(eb.y << 16), __uint_as_float(eb.y & 0xffff0000u)};
          resid_store<MT, MP, PL::xn>(p, hn, m, n, lane, *(const gu32x2*)(L.attn_norm + n), p.h, p.xn, p.ssq, u);
        }
      }
    } else if (sub == 0 || sub == 3 || sub == 5) {
      // one instance of the loop for the three phases where their operands have the same number of planes (the code
      // has to stay resident in the instruction cache across the layers)
      bool ok;
      if constexpr (PL::xn == PL::att && PL::xn == PL::act) {
        ok = gemm_phase<kAtQkv, MT, PL::xn, 2, true, MP, PL::xn, PL::act>(p, g, bsrc, bplane, epi, e, grid, do_wait, red, r_s, ssq_in, ph, my_unit);
      } else {
        if (sub == 0) ok = gemm_phase<kAtQkv, MT, PL::xn, 2, true, MP, PL::xn, PL::act>(p, g, bsrc, bplane, epi, e, grid, do_wait, red, r_s, ssq_in, ph, my_unit);
        else if (sub == 3) ok = gemm_phase<kAtQkv, MT, PL::att, 2, true, MP, PL::xn, PL::act>(p, g, bsrc, bplane, epi, e, grid, do_wait, red, r_s, ssq_in, ph, my_unit);
        else ok = gemm_phase<kAtQkv, MT, PL::act, 2, true, MP, PL::xn, PL::act>(p, g, bsrc, bplane, epi, e, grid, do_wait, red, r_s, ssq_in, ph, my_unit);
      }
      if (!ok) return;
      // (the unit's stores have left: it ended with a drain and a workgroup barrier)
      if (qkv_flag >= 0 && threadIdx.x == 0)
        __hip_atomic_store(p.qkv_flags + qkv_flag, grid.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else if (sub == 4 || sub == 6) {
      const bool ok = gemm_phase<4, MT, PL::xn, Depth<MT, DEEP, PL::xn>::a4, false, MP, PL::xn, PL::act>(p, g, bsrc, bplane, epi, e, grid, do_wait, red, r_s, ssq_in, ph, my_unit);
      if (!ok) return;
      if (sub == 6 && p.hidden) {
        // final-norm hidden states (the row scales are in LDS)
        const gfloat* hv = (const gfloat*)(p.h + (int64_t)(2 * p.L) * h_stride);
        for (int m = blockIdx.x; m < p.M; m += p.nwg)
          for (int c = threadIdx.x; c < p.d; c += kFusedThreads)
            p.hidden[(int64_t)m * p.hidden_ld + c] = hv[(int64_t)m * p.d + c] * bf16_to_f32(p.final_norm[c]) * r_s[m];
      }
    } else if (sub == 1) {
      float* part_o = p.part_o + (int64_t)l * p.part_layer_stride * 64;
      float* part_ml = p.part_ml + (int64_t)l * p.part_layer_stride * 2;
      // the qkv phase left this layer's row scales in LDS; a launch that starts here computes them itself
      if (ph == first) compute_row_scales<MP>(p, p.ssq + (int64_t)(2 * l) * ssq_stride, r_s);
      // a workgroup with a unit waits for the grid inside its first unit, after requesting that unit's stored keys
      const bool group = gs && ph > first;           // wait for the unit's group instead of the grid
      bool waited = !(do_wait || group);
      for (int u = p.nwg - 1 - (int)blockIdx.x; u < p.n_attn_units; u += p.nwg) {
        if (!attn_unit<MT, MP, PL::q, PL::p, PL::att, PG, SM>(p, L, qkv, u, r_s, red, att, part_o, part_ml,
                                                           p.arrivals + (int64_t)l * p.arrivals_stride, ph, waited ? nullptr : &grid,
                                                           group ? p.qkv_flags + l * 128 : nullptr)) return;
        waited = true;
      }
      if (!waited && !group) {
        if (!grid_wait(grid)) return;
        stamp(p, ph, 1);
      }
    } else {
      // merge of the key splits; with a single split the attention units wrote the final output and this phase
      // (and its barrier) does not exist
      float* part_o = p.part_o + (int64_t)l * p.part_layer_stride * 64;
      float* part_ml = p.part_ml + (int64_t)l * p.part_layer_stride * 2;
      if (do_wait && !grid_wait(grid)) return;
      stamp(p, ph, 1);
      for (int u = blockIdx.x; u < p.n_pair_units; u += p.nwg) attn_merge_unit<MT, MP, PL::att>(p, u, part_o, part_ml, att);
    }
    stamp(p, ph, 2);
    if (ph < last && !(gs && sub == 0)) grid_arrive(grid);
  }
  // every workgroup read the word before the first barrier of this launch, which workgroup 0 has passed by now
  if (persistent && blockIdx.x == 0 && threadIdx.x == 0) p.bar[kBarEpochWord] = grid.epoch;
}

// ---------------------------------------------------------------------------------------------- set-up kernels
__global__ void retile_stream_kernel(const bf16_t* __restrict__ src0, int rows0, const bf16_t* __restrict__ src1, int rows1,
                                     const bf16_t* __restrict__ src2, int rows2, int mode, int AT, int KS, int Kd, int n_units,
                                     bf16_t* __restrict__ dst) {
  const int KTW = Kd / 32 / kFusedWaves / KS;
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
  const int64_t unit = tile / kFusedWaves;
  const int64_t u = unit / KS;            // feature-tile group
  const int ks = (int)(unit % KS);        // k-slice
  const int kt = (ks * kFusedWaves + w) * KTW + i;
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

// [B][len][Hkv][64] keys and values -> the head-major trunk layouts of the fused pass
// pages != null: paged trunk, block j of sequence b in page pages[b * page_stride + j] of the pool
__global__ void copy_kv_fused_kernel(bf16_t* trunk_k, bf16_t* trunk_vt, const bf16_t* src_k, const bf16_t* src_v, int len,
                                     int Hkv, int vt_stride, int64_t total, const int32_t* pages, int page_stride) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // over [B][len][Hkv][64]
  if (idx >= total) return;
  int d = (int)(idx & 63);
  int64_t r = idx >> 6;
  int hk = (int)(r % Hkv);
  r /= Hkv;
  int pos = (int)(r % len);
  int64_t b = r / len;
  const int64_t bb = pages ? ((int64_t)pages[b * page_stride + (pos >> 5)] * Hkv + hk) * 2048
                           : (b * Hkv + hk) * (int64_t)vt_stride * 64 + (int64_t)(pos >> 5) * 2048;
  trunk_k[bb + (int64_t)(pos & 31) * 64 + d] = src_k[idx];
  trunk_vt[bb + d * 32 + (pos & 31)] = src_v[idx];
}

constexpr size_t kFusedLdsBytes = 96 * 1024;   // reduction tiles (<= 8 wavefronts x 12 tiles x 1 KiB); also keeps one workgroup per CU

template <int MT, bool DEEP, class PL, bool PG, bool SM>
int check_residency_sm(int nwg, int cus) {
  SSD_HIP(hipFuncSetAttribute((const void*)fused_kernel<MT, DEEP, PL, PG, SM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedLdsBytes));
  int per_cu = 0;
  SSD_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fused_kernel<MT, DEEP, PL, PG, SM>, kFusedThreads, kFusedLdsBytes));
  SSD_CHECK_ARG((int64_t)per_cu * cus >= nwg,
                "fused pass: %d workgroups cannot be resident at once (%d per compute unit x %d compute units): the grid barrier "
                "would never complete", nwg, per_cu, cus);
  return SSD_OK;
}

template <int MT, bool DEEP, class PL, bool PG>
int check_residency_mt(int nwg, int cus) {
  SSD_TRY((check_residency_sm<MT, DEEP, PL, PG, false>(nwg, cus)));
  return check_residency_sm<MT, DEEP, PL, PG, true>(nwg, cus);
}

template <int MT, bool DEEP, class PL, bool PG, bool SM>
int launch_sm(const FusedParams& p, int first, int last, int persistent, hipStream_t s) {
  const size_t lds = kFusedLdsBytes;
  static bool configured = false;
  if (!configured) {
    SSD_HIP(hipFuncSetAttribute((const void*)fused_kernel<MT, DEEP, PL, PG, SM>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    configured = true;
  }
  if (persistent) {
    fused_kernel<MT, DEEP, PL, PG, SM><<<p.nwg, kFusedThreads, lds, s>>>(p, first, last, 1);
    SSD_HIP(hipGetLastError());
  } else {
    const int lm_phase = fused_last_phase(p.L);
    for (int ph = first; ph <= last; ++ph) {
      if ((SM || p.NS == 1) && ph > 0 && ph < lm_phase && (ph - 1) % 6 == 2) continue;   // no merge phase
      fused_kernel<MT, DEEP, PL, PG, SM><<<p.nwg, kFusedThreads, lds, s>>>(p, ph, ph, 0);
      SSD_HIP(hipGetLastError());
    }
  }
  return SSD_OK;
}

// Passes with several key splits take the kernel whose attention units merge them.
template <int MT, bool DEEP, class PL, bool PG>
int launch_mt(const FusedParams& p, int first, int last, int persistent, hipStream_t s) {
  if (p.NS > 1) return launch_sm<MT, DEEP, PL, PG, true>(p, first, last, persistent, s);
  return launch_sm<MT, DEEP, PL, PG, false>(p, first, last, persistent, s);
}

}  // namespace

int64_t stream_order_elems(int N, int Kd, int AT) {
  int64_t nt = (N + 15) / 16;
  int64_t units = (nt + AT - 1) / AT;
  return units * AT * 16 * (int64_t)Kd;
}

int launch_retile_stream(const bf16_t* src0, int rows0, const bf16_t* src1, int rows1, const bf16_t* src2, int rows2,
                         int mode, int AT, int KS, int Kd, bf16_t* dst, hipStream_t s) {
  SSD_CHECK_ARG(KS >= 1 && Kd % (256 * KS) == 0, "fused path: reduction dimension %d must be a multiple of %d", Kd, 256 * KS);
  SSD_CHECK_ARG(mode == 0 || (AT == 4 && rows0 == rows1 && rows0 % 32 == 0), "gate/up interleave needs AT = 4 and equal heights");
  int64_t nt = mode == 0 ? ((int64_t)rows0 + rows1 + rows2 + 15) / 16 : (int64_t)2 * (rows0 / 16);
  int n_units = (int)((nt + AT - 1) / AT) * KS;
  int64_t total = (int64_t)(n_units / KS) * AT * (Kd / 32) * 64;
  retile_stream_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(src0, rows0, src1, rows1, src2, rows2, mode, AT, KS, Kd,
                                                                       n_units, dst);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

// A stream-order weight buffer from bf16 to fp16: same layout, every element converted (8 per thread)
__global__ void bf16_to_f16_kernel(const bf16_t* src, bf16_t* dst, int64_t n8) {   // dst may be src
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n8) return;
  Bf8 v, o;
  v.w = *(const u32x4*)(src + i * 8);
#pragma unroll
  for (int e = 0; e < 8; ++e) o.u[e] = to_f16(bf16_to_f32(v.u[e]));
  *(u32x4*)(dst + i * 8) = o.w;
}

int launch_bf16_to_f16(const bf16_t* src, bf16_t* dst, int64_t n, hipStream_t s) {
  SSD_CHECK_ARG(n % 8 == 0, "bf16_to_f16: element count %lld is not a multiple of 8", (long long)n);
  if (n == 0) return SSD_OK;
  bf16_to_f16_kernel<<<(unsigned)((n / 8 + 255) / 256), 256, 0, s>>>(src, dst, n / 8);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

int launch_copy_kv_fused(bf16_t* trunk_k, bf16_t* trunk_vt, const bf16_t* src_k, const bf16_t* src_v, int B, int len, int Hkv,
                         int vt_stride, const int32_t* pages, int page_stride, hipStream_t s) {
  int64_t total = (int64_t)B * len * Hkv * 64;
  if (total == 0) return SSD_OK;
  copy_kv_fused_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(trunk_k, trunk_vt, src_k, src_v, len, Hkv, vt_stride, total, pages, page_stride);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

bool fused_supported(const Dims& d, int max_rows) {
  return d.dtype == SSD_BF16 && d.head_dim == 64 && max_rows <= kFusedMaxRows && d.d_model % 512 == 0 &&
         d.q_dim() % 512 == 0 && d.d_ffn % 512 == 0 && d.kv_dim() % 16 == 0 && d.vocab % 16 == 0 &&
         d.n_q_heads % d.n_kv_heads == 0 && 16 % (d.n_q_heads / d.n_kv_heads) == 0;
}

int fused_init_barrier(unsigned* bar, unsigned epoch0, int nwg) {
  static_assert(kBarEpochWord < kFusedSyncWords && kBarFlags + kBarGroups <= kFusedSyncWords, "barrier words");
  std::vector<unsigned> w(kFusedSyncWords + 64, 0u);
  for (int g = 0; g < kBarGroups; ++g) {
    w[32 * g] = epoch0 * (unsigned)(nwg / kBarGroups);   // arrivals so far, modulo 2^32 like the counter itself
    w[kBarFlags + g] = epoch0;
  }
  w[kBarEpochWord] = epoch0;
  SSD_HIP(hipMemcpy(bar, w.data(), w.size() * sizeof(unsigned), hipMemcpyHostToDevice));
  return SSD_OK;
}

int fused_init_group_flags(unsigned* flags, int n_layers, unsigned epoch0) {
  std::vector<unsigned> w((size_t)n_layers * 128, epoch0);
  SSD_HIP(hipMemcpy(flags, w.data(), w.size() * sizeof(unsigned), hipMemcpyHostToDevice));
  return SSD_OK;
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

// The plane configurations that are compiled in: bit i of the mask set = that tensor travels as ONE plane
// (bit 0 xn, 1 att, 2 act, 3 q, 4 p).  The default, and the only one with a paged trunk: xn, att, act one fp16 plane,
// q and p two bf16 planes (what the second plane of the former costs a 24-row step of the 1B shape: 4 %; 11 % at 48 rows
// and 8192 keys; the error against a float64 reference goes from 1.1e-3 to 2.6e-3).
constexpr int kFusedDefaultPlanes = 7;
#ifndef SSD_FUSED_PLANE_MASKS
#define SSD_FUSED_PLANE_MASKS X(0) X(7)
#endif
template <int MASK>
using PlanesOf = Planes<(MASK & 1) ? 1 : 2, (MASK & 2) ? 1 : 2, (MASK & 4) ? 1 : 2, (MASK & 8) ? 1 : 2, (MASK & 16) ? 1 : 2>;

template <class PL, bool PG>
int check_residency_pl(int nwg, int cus) {
  SSD_TRY((check_residency_mt<1, true, PL, PG>(nwg, cus)));
  SSD_TRY((check_residency_mt<2, true, PL, PG>(nwg, cus)));
  SSD_TRY((check_residency_mt<3, true, PL, PG>(nwg, cus)));
  SSD_TRY((check_residency_mt<1, false, PL, PG>(nwg, cus)));
  SSD_TRY((check_residency_mt<2, false, PL, PG>(nwg, cus)));
  SSD_TRY((check_residency_mt<3, false, PL, PG>(nwg, cus)));
  return SSD_OK;
}

template <int ATW, int EPI, int D, int MTG>
int launch_wide_gemm_dm(const FusedParams& p, const FusedGemm& g, const bf16_t* bsrc, const WideEpi& e, hipStream_t s) {
  static bool configured = false;
  if (!configured) {
    SSD_HIP(hipFuncSetAttribute((const void*)wide_gemm_kernel<ATW, EPI, D, MTG>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedLdsBytes));
    configured = true;
  }
  wide_gemm_kernel<ATW, EPI, D, MTG><<<p.nwg, kWideThreads, kFusedLdsBytes, s>>>(p, g, bsrc, e);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

template <int ATW, int EPI, int D>
int launch_wide_gemm_d(const FusedParams& p, const FusedGemm& g, const bf16_t* bsrc, const WideEpi& e, hipStream_t s) {
  // Row groups as small as still give every pair a workgroup of its own: what bounds these kernels is what one compute
  // unit pulls (4 KiB of weights + 1 KiB per row tile of the group, per k-tile), and with few rows or few feature tiles
  // the full-size groups leave most of the grid without a pair while the busy workgroups pull as much as ever.
  const int nq = ATW == 4 ? g.n_units / g.KS : (g.n_units / g.KS) >> 1;
  const int tiles = (p.M + 15) >> 4;
  auto fits = [&](int mtg) { return nq * ((tiles + mtg - 1) / mtg) <= p.nwg; };
  if constexpr (ATW == 2) {
    if (fits(1)) return launch_wide_gemm_dm<ATW, EPI, D, 1>(p, g, bsrc, e, s);
    if (fits(2)) return launch_wide_gemm_dm<ATW, EPI, D, 2>(p, g, bsrc, e, s);
    if (fits(kWideGroup / 2)) return launch_wide_gemm_dm<ATW, EPI, D, kWideGroup / 2>(p, g, bsrc, e, s);
  }
  return launch_wide_gemm_dm<ATW, EPI, D, kWideGroup>(p, g, bsrc, e, s);
}

template <int EPI>
int launch_wide_gemm_lds(const FusedParams& p, const FusedGemm& g, const bf16_t* bsrc, const WideEpi& e, hipStream_t s) {
  static bool configured = false;
  if (!configured) {
    SSD_HIP(hipFuncSetAttribute((const void*)wide_gemm_lds_kernel<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedLdsBytes));
    configured = true;
  }
  wide_gemm_lds_kernel<EPI><<<p.nwg, kWideThreads, kFusedLdsBytes, s>>>(p, g, bsrc, e);
  SSD_HIP(hipGetLastError());
  return SSD_OK;
}

template <int ATW, int EPI>
int launch_wide_gemm(const FusedParams& p, const FusedGemm& g, const bf16_t* bsrc, const WideEpi& e, hipStream_t s) {
  // a wavefront's k-tiles per pair must be whole turns of the ring
  if ((2 * g.KS * g.KTW) % kWideRing == 0) return launch_wide_gemm_d<ATW, EPI, kWideRing>(p, g, bsrc, e, s);
  return launch_wide_gemm_d<ATW, EPI, kWideRing / 2>(p, g, bsrc, e, s);
}

// One wide pass: phases [first, last] as one launch each.  layers_host: the pass's layer table in host memory.
template <class PL, bool PG>
int launch_wide_pl(const FusedParams& p, const FusedLayer* layers_host, int first, int last, hipStream_t s) {
  static bool configured = false;
  if (!configured) {
    SSD_HIP(hipFuncSetAttribute((const void*)wide_kernel<PL, PG>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedLdsBytes));
    configured = true;
  }
  constexpr int64_t MP = kFusedWideRows;
  const int64_t h_stride = MP * p.d, ssq_stride = (int64_t)(p.d >> 4) * MP;
  const int lm_phase = fused_last_phase(p.L);
  for (int ph = first; ph <= last; ++ph) {
    const int l = ph == 0 ? 0 : (ph == lm_phase ? p.L - 1 : (ph - 1) / 6);
    const int sub = ph == 0 ? -1 : (ph == lm_phase ? 6 : (ph - 1) % 6);
    if (sub == 2 && p.NS == 1) continue;             // no merge phase with one key split
    const FusedLayer& L = layers_host[l];
    float* qkv = p.qkv + (int64_t)l * MP * p.qkvd;
    bf16_t* att = p.att + (int64_t)l * 2 * MP * p.qd;
    bf16_t* act = p.act + (int64_t)l * 2 * MP * p.ffn;
    WideEpi e{};
    e.ph = ph;
    if (sub == 0) {
      e.out = qkv; e.ld = p.qkvd; e.ssq_in = p.ssq + (int64_t)(2 * l) * ssq_stride;
      SSD_TRY((launch_wide_gemm<2, FE_QKV>(p, L.qkv, p.xn + (int64_t)(2 * l) * 2 * h_stride, e, s)));
    } else if (sub == 3 || sub == 5) {
      const int v = sub == 3 ? 2 * l + 1 : 2 * l + 2;
      e.h_in = p.h + (int64_t)(v - 1) * h_stride;
      e.h_out = p.h + (int64_t)v * h_stride;
      e.gain = sub == 3 ? L.mlp_norm : (l + 1 < p.L ? layers_host[l + 1].attn_norm : p.final_norm);
      e.xn_out = p.xn + (int64_t)v * 2 * h_stride;
      e.ssq_out = p.ssq + (int64_t)v * ssq_stride;
      SSD_TRY((launch_wide_gemm<2, FE_RESID>(p, sub == 3 ? L.o : L.down, sub == 3 ? att : act, e, s)));
    } else if (sub == 4) {
      const int v = 2 * l + 1;
      e.act_out = act; e.ssq_in = p.ssq + (int64_t)v * ssq_stride;
      // one row group (up to 96 rows): a workgroup per unit of 4 feature tiles, the reduction dimension over its
      // wavefronts, instead of 16 feature tiles per workgroup on a quarter of the grid
      if (((p.M + 15) >> 4) <= kWideGroup && L.gu.n_units <= p.nwg) {
        SSD_TRY((launch_wide_gemm<4, FE_SWIGLU>(p, L.gu, p.xn + (int64_t)v * 2 * h_stride, e, s)));
      } else {
        SSD_TRY((launch_wide_gemm_lds<FE_SWIGLU>(p, L.gu, p.xn + (int64_t)v * 2 * h_stride, e, s)));
      }
    } else {
      if (sub == 6 && p.logits) {
        const int v = 2 * p.L;
        e.out = p.logits; e.ld = p.logits_ld; e.ssq_in = p.ssq + (int64_t)v * ssq_stride;
        SSD_TRY((launch_wide_gemm_lds<FE_LOGITS>(p, p.lm, p.xn + (int64_t)v * 2 * h_stride, e, s)));
      }
      if (sub == 6 && !p.hidden) continue;
      int grid = p.nwg;
      if (sub == 1) grid = p.n_attn_units;
      else if (sub == 2) grid = p.n_pair_units;
      else if (sub == 6) grid = p.M;
      wide_kernel<PL, PG><<<grid, kFusedThreads, kFusedLdsBytes, s>>>(p, ph);
      SSD_HIP(hipGetLastError());
    }
  }
  return SSD_OK;
}

template <class PL, bool PG>
int launch_pl(const FusedParams& p, int first, int last, int persistent, hipStream_t s) {
  const int mt = (p.M + 15) / 16;
  if (p.deep != 0) {
    if (mt == 1) return launch_mt<1, true, PL, PG>(p, first, last, persistent, s);
    if (mt == 2) return launch_mt<2, true, PL, PG>(p, first, last, persistent, s);
    return launch_mt<3, true, PL, PG>(p, first, last, persistent, s);
  }
  if (mt == 1) return launch_mt<1, false, PL, PG>(p, first, last, persistent, s);
  if (mt == 2) return launch_mt<2, false, PL, PG>(p, first, last, persistent, s);
  return launch_mt<3, false, PL, PG>(p, first, last, persistent, s);
}

bool fused_planes_supported(int mask) {
#define X(m) if (mask == (m)) return true;
  SSD_FUSED_PLANE_MASKS
#undef X
  return false;
}

int fused_check_residency(int nwg, int planes, int paged) {
  int dev = 0, cus = 0;
  SSD_HIP(hipGetDevice(&dev));
  SSD_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  if (paged) {
    SSD_CHECK_ARG(planes == kFusedDefaultPlanes, "a paged trunk takes the default activation planes only");
    return check_residency_pl<PlanesOf<kFusedDefaultPlanes>, true>(nwg, cus);
  }
#define X(m) if (planes == (m)) return check_residency_pl<PlanesOf<(m)>, false>(nwg, cus);
  SSD_FUSED_PLANE_MASKS
#undef X
  set_error("fused pass: plane configuration %d is not compiled in", planes);
  return SSD_EINVAL;
}

// Wide passes carry xn, att and act as ONE fp16 plane each (2.5e-3 between hidden states and a float64 reference through
// 16 layers, measured); the attention unit's queries and probabilities keep two bf16 planes unless both of their bits
// are set in p.planes.
int launch_fused_wide(const FusedParams& p, const FusedLayer* layers_host, int first, int last, hipStream_t s) {
  SSD_CHECK_ARG(p.M >= 1 && p.M <= kFusedWideRows, "wide fused pass of %d rows (1..%d supported)", p.M, kFusedWideRows);
  SSD_CHECK_ARG(p.nwg >= 8 && p.nwg % 8 == 0, "fused grid of %d workgroups must be a multiple of 8", p.nwg);
  SSD_CHECK_ARG(p.KPU >= 32 && p.KPU % 32 == 0 && p.NS >= 1 && p.QT >= 1 && (p.SL == 8 || p.SL == 16) && 16 % p.G == 0 &&
                    (16 / p.G) * p.SL <= 64,
                "bad attention split");
  SSD_CHECK_ARG(first >= 0 && last <= fused_last_phase(p.L) && first <= last && layers_host, "bad phase range");
  if (p.pages) {
    SSD_CHECK_ARG((p.planes & 24) != 24, "a paged trunk takes the default planes of the attention unit only");
    return launch_wide_pl<Planes<1, 1, 1, 2, 2>, true>(p, layers_host, first, last, s);
  }
  if ((p.planes & 24) == 24) return launch_wide_pl<Planes<1, 1, 1, 1, 1>, false>(p, layers_host, first, last, s);
  return launch_wide_pl<Planes<1, 1, 1, 2, 2>, false>(p, layers_host, first, last, s);
}

// Shapes the wide pass takes: every layer's stream-order layout must cut into sets of 4 feature tiles over whole
// k-ranges of an even number of k-tiles per wavefront.
bool fused_wide_gemm_ok(const FusedGemm& g, int at) {
  if ((2 * g.KS * g.KTW) % (kWideRing / 2)) return false;     // a wavefront's k-tiles per pair, in whole turns of the (half) ring
  if (at == 4) return g.KS == 1;
  return at == 2 && (g.n_units / g.KS) % 2 == 0;
}

int launch_fused(const FusedParams& p, int first, int last, int persistent, hipStream_t s) {
  SSD_CHECK_ARG(p.M >= 1 && p.M <= kFusedMaxRows, "fused pass of %d rows (1..%d supported)", p.M, kFusedMaxRows);
  SSD_CHECK_ARG(p.nwg >= 8 && p.nwg % 8 == 0, "fused grid of %d workgroups must be a multiple of 8", p.nwg);
  SSD_CHECK_ARG(p.KPU >= 32 && p.KPU % 32 == 0 && p.NS >= 1 && p.QT >= 1 && (p.SL == 8 || p.SL == 16) && 16 % p.G == 0 &&
                    (16 / p.G) * p.SL <= 64,
                "bad attention split");
  SSD_CHECK_ARG(first >= 0 && last <= fused_last_phase(p.L) && first <= last, "bad phase range");
  SSD_CHECK_ARG(p.NS <= 16 && (p.NS == 1 || p.arrivals), "fused pass: %d key splits (at most 16, with arrival counters)", p.NS);
  SSD_CHECK_ARG(p.qkv_ug == 0 || (p.qkv_flags && p.qkv_ug <= 16 && p.qkv_ug == 2 * p.G + 4 && p.Hkv <= 8 && 8 % p.Hkv == 0 &&
                                  8 * p.qkv_ug <= p.nwg && (!persistent || first == 0)),
                "fused pass: group sync does not fit this shape or phase range");
  if (p.pages) {
    SSD_CHECK_ARG(p.planes == kFusedDefaultPlanes, "a paged trunk takes the default activation planes only");
    return launch_pl<PlanesOf<kFusedDefaultPlanes>, true>(p, first, last, persistent, s);
  }
#define X(m) if (p.planes == (m)) return launch_pl<PlanesOf<(m)>, false>(p, first, last, persistent, s);
  SSD_FUSED_PLANE_MASKS
#undef X
  set_error("fused pass: plane configuration %d is not compiled in", p.planes);
  return SSD_EINVAL;
}

}  // namespace ssd
