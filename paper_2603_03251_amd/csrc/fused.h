// The fused decode pass for bf16 models with few rows (M <= 48): one batched forward of the draft decoder
// (embedding, every layer, LM head) as ONE persistent kernel of one workgroup per compute unit.  Phases are
// separated by a grid barrier; workgroups exchange activations through memory that is written once per launch
// (write-through stores, plain loads), and each workgroup issues the weight loads of its next phase before it
// waits at the barrier, so the weight stream keeps running across phase boundaries.
// Shared between the round driver (ssd_api.hip) and kernels_fused.hip.
#pragma once

#include "common.h"

namespace ssd {

constexpr int kFusedThreads = 512;  // 8 wavefronts; they split the reduction dimension of a weight block
constexpr int kFusedWaves = 8;
constexpr int kFusedMaxRows = 48;   // rows of one narrow pass (three 16-row MFMA tiles)
constexpr int kFusedWideRows = 384; // rows of one wide pass (24 row tiles): contexts with more than kFusedMaxRows rows
constexpr int kFusedWideQueryTiles = 3;   // wide passes: query tiles per attention unit (n_attn_units counts such units)
constexpr int kFusedClockSlots = 8;  // clock probes per phase and workgroup (see stamp())
constexpr int kFusedMaxSlices = 4;   // most k-slices of a linear layer
constexpr unsigned kFusedSpinLimit = 4000000u;   // polls of a bounded wait (seconds of wall time) before it gives up

// A linear layer in "stream order".  The [N][Kd] matrix is cut into 1 KiB MFMA tiles (16 features x 32 inputs,
// stored as the 64 lanes of an MFMA 16x16x32 A operand hold them).  A unit is AT feature tiles over the whole
// reduction dimension; inside a unit wavefront w owns the k-tiles w*KTW .. w*KTW+KTW-1.  Tiles are stored
// [unit][wavefront][k-tile of the wavefront][feature tile of the unit], so each wavefront streams one contiguous
// run of memory per unit.  Workgroup g takes units g, g + grid, ...
struct FusedGemm {
  const bf16_t* w;  // 16-bit elements holding fp16 (converted from the model's bf16 when the layout is built)
  int KTW;      // k-tiles per wavefront and unit = Kd / 32 / 8 / KS
  int n_units;  // ceil(NT / AT) * KS
  int NT;       // real feature tiles (the last unit may hold zero padding)
  int KS;       // k-slices (<= kFusedMaxSlices): with KS > 1 unit u = (tile group u / KS, slice u % KS) covers 1/KS of the
                // reduction dimension and slice 0 adds the others' partial tiles in order; needs n_units <= grid
};

struct FusedLayer {
  FusedGemm qkv, o, gu, down;              // gu: unit p = gate tiles 2p, 2p+1 then up tiles 2p, 2p+1
  const bf16_t *attn_norm, *mlp_norm;      // gains [d]
  bf16_t *trunk_k;                         // [B][Hkv][vt_stride][64]              (head-major)
  bf16_t *trunk_vt;                        // [B][Hkv][vt_stride / 32][64][32]     (values transposed per 32-key block)
  bf16_t *suffix_k, *suffix_v;             // [M][suffix_cap][Hkv][64]
};

struct FusedParams {
  // model
  int L, d, qd, kvd, qkvd, ffn, V, Hq, Hkv, G;
  float eps;
  const FusedLayer* layers;                // device array [L]
  const bf16_t *embed, *final_norm;
  FusedGemm lm;
  // this pass
  int M, B, R;                             // rows, sequences, rows per sequence (rows of a sequence are consecutive)
  const RowDesc* rows;
  const float* cos_sin;                    // [M][32][2]
  const int32_t* tokens;
  int max_trunk, vt_stride, suffix_cap;
  // paged trunk (null: contiguous): block j (32 positions) of sequence b of this pass is page pages[b * page_stride + j]
  // of the pool every layer's trunk_k / trunk_vt point at ([page][Hkv][32][64] keys, [page][Hkv][64][32] values);
  // page 0 is never handed out and holds zeros
  const int32_t* pages;
  int page_stride;
  // attention work split: unit = (sequence, KV head, 16-row query tile, key split)
  int KPU;                                 // stored trunk keys per split (multiple of 32)
  int NS;                                  // key splits; 1 = the attention phase writes the final output
  int QT;                                  // query tiles per (sequence, KV head) = ceil(R G / 16)
  int SL;                                  // fresh-key slots per branch row (8 or 16)
  int is_branch;                           // 1: branch rows (private suffix), 0: extend rows (causal among themselves)
  int suffix_len;                          // branch rows: private positions a row sees, its own token included
  int tv_ub;                               // host bound of the stored trunk keys any row sees (loop counts only)
  int n_attn_units, n_pair_units;          // B Hkv QT NS attention units; ceil(M Hq / 8) merge units (wide passes)
  // workspace, every address written at most once per launch
  float* h;        // [2L+1][48][d]    residual stream after embed / each o-proj / each down-proj
  bf16_t* xn;      // [2L+1][2][48*d]  (h * gain of the next norm) as fp16 planes (head, remainder) in B-operand order
  float* ssq;      // [2L+1][d/16][48] per-feature-tile partial sums of h^2
  float* qkv;      // [L][48][qkvd]    raw projections (before the norm's row scale and the rotary embedding)
  bf16_t* att;     // [L][2][48*qd]    attention output planes, B-operand order
  bf16_t* act;     // [L][planes][48*ffn]
  float* fix_buf;  // [L][3][fix_stride]  partial tiles of K-split linear layers (qkv, o, down); every word holds
                   // 0xffffffff ("not written yet") between launches: the reader of a tile puts that value back
  int64_t fix_stride;
  float* part_o;   // [L][B][Hkv][NS][QT*16][64]  partial softmaxes of the key splits (NS > 1 only)
  float* part_ml;  // [L][B][Hkv][NS][QT*16][2]
  unsigned* qkv_flags;      // [L][8][16]: per layer and KV head, the barrier number at which each qkv unit of that head's
  int qkv_ug;               // group was stored (group sync of the narrow persistent pass); units per group, 0 = off
  unsigned* arrivals;       // [L][arrivals_stride]: per (sequence, KV head, query tile) the key splits that have stored their
  int64_t arrivals_stride;  // partial softmax in this pass; zero between passes (the last arrival merges and resets)
  int64_t part_layer_stride;               // in (q-row) entries
  float* logits;   int64_t logits_ld;      // may be null
  float* hidden;   int64_t hidden_ld;      // may be null
  unsigned* bar;                           // 2048 grid-barrier words, zeroed once; epochs carry over between launches
  unsigned* err;                           // set to 1 if a bounded wait expired (host-pinned memory: the host reads it
                                           // without synchronising)
  unsigned spin_limit;                     // polls a bounded wait may take before it gives up
  unsigned long long* prof;                // optional [phases][kFusedClockSlots][nwg] real-time-counter ticks, or null
  int nwg;
  int deep;                                // 1: every linear layer has a multiple of 4 k-tiles per wavefront and unit
  int planes;                              // bit i set: tensor i travels as one 16-bit plane instead of head + remainder
                                           // (0 xn, 1 att, 2 act, 3 q, 4 p); see Planes in kernels_fused.hip
};

// Phase ids: 0 embed; 1 + 6 l + {0 qkv, 1 attention, 2 merge of key splits (NS > 1 only), 3 o-proj, 4 gate/up, 5 down};
// 1 + 6 L LM head.
__host__ __device__ inline int fused_last_phase(int L) { return 1 + 6 * L; }

// Retile row-major bf16 matrices into stream order.  `mode` 0: rows of src0, src1, src2 concatenated along the
// feature dimension (rows0, rows1, rows2 features); mode 1: gate/up interleave (src0 = gate, src1 = up, AT = 4).
int launch_retile_stream(const bf16_t* src0, int rows0, const bf16_t* src1, int rows1, const bf16_t* src2, int rows2,
                         int mode, int AT, int KS, int Kd, bf16_t* dst, hipStream_t s);
int64_t stream_order_elems(int N, int Kd, int AT);
// [B][len][Hkv][64] keys and values -> the trunk layouts of FusedLayer
int launch_copy_kv_fused(bf16_t* trunk_k, bf16_t* trunk_vt, const bf16_t* src_k, const bf16_t* src_v, int B, int len, int Hkv,
                         int vt_stride, const int32_t* pages, int page_stride, hipStream_t s);

// feature tiles per unit of each linear layer
constexpr int kAtQkv = 2, kAtO = 2, kAtGu = 4, kAtDown = 2, kAtLm = 4;

bool fused_supported(const Dims& d, int max_rows);
// Runs phases [first, last].  persistent = 1: one launch with grid barriers between phases;
// persistent = 0: one launch per phase (a debugging aid that needs no co-residency).
int launch_fused(const FusedParams& p, int first, int last, int persistent, hipStream_t s);
// The same phases for up to kFusedWideRows rows (workspace strides of kFusedWideRows rows, one fp16 plane per tensor),
// one launch per phase.  layers_host: the layer table p.layers points at, in host memory.
int launch_fused_wide(const FusedParams& p, const FusedLayer* layers_host, int first, int last, hipStream_t s);
bool fused_wide_gemm_ok(const FusedGemm& g, int at);
// dst[i] = fp16(src[i]) over a stream-order weight buffer (the fused passes multiply in fp16; dst may be src); n a multiple of 8
int launch_bf16_to_f16(const bf16_t* src, bf16_t* dst, int64_t n, hipStream_t s);
int fused_grid_size(int* out);
// EINVAL unless `nwg` workgroups of every instance of the persistent kernel can be resident at once on the current device
int fused_check_residency(int nwg, int planes, int paged);
bool fused_planes_supported(int planes);
// Barrier words (kFusedSyncWords of them + the error word behind) as a finished barrier number `epoch0` leaves them;
// 0 for a new context.  The epoch counts on from launch to launch and wraps after 2^32 barriers.
constexpr int kFusedSyncWords = 2048;
int fused_init_barrier(unsigned* bar, unsigned epoch0, int nwg);
// the group-sync flags as that barrier number leaves them (no qkv unit of a coming launch carries it)
int fused_init_group_flags(unsigned* flags, int n_layers, unsigned epoch0);

}  // namespace ssd
