// Internal declarations shared by the translation units of libdsmoe (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/dsmoe.h"

namespace dsmoe {

constexpr int kMaxTopK = 16;
constexpr int kMaxExperts = 512;
constexpr int kMaxPart = 8;
constexpr int kSubBits = 4;  // partitions that take part in the row sort key
constexpr int kSplitItems = 256;  // one GEMM-2 item per compute unit: the granularity K splits aim at (measured best)
constexpr int kMaxSplit = 8;      // most K ranges an item is split into when there are few row tiles (decode-sized batches)
constexpr int kTallExtra = 64;    // rows beyond a full tile that a tall GEMM item takes along
constexpr int kPoolRows = 256 + kTallExtra;  // rows of a partial-output tile of the pool (kMfmaBM + kTallExtra)
constexpr int kSplitRowsOffset = 1 << 30;    // flag in the (row tile, column tile) -> pool tile table: the tile's rows sit kMfmaBM rows down
constexpr int kMaxTailSplit = 8;  // most K ranges an item of the last, partly filled round of items is split into
constexpr int kPoolTiles = 768;   // partial-output tiles (256 x 256) the extra K ranges can need at most
// Half-precision partial outputs hold the GEMM-2 accumulators times 2^-10.  The accumulators are sums
// over the kept neurons of (activation x 2^k) x (W2 x 2^s) with the largest |W2 x 2^s| in [2^14, 2^15):
// for activations of order one they are of order sqrt(neurons) x 5000, i.e. 1e2 .. 1e3 after the
// scaling, with a factor 60 and more up to half precision's largest value and seven decades down to its
// smallest normal one, whatever the scale of the weights (and, through cfg.h_scale_log2, of the activations).
constexpr float kYpHalfScale = 1.0f / 1024.0f;
constexpr int kSelBins = 4096;  // grid of the row-budget thresholds: multiples of 2^-12 (a power of two keeps n * kSelBins exact)
constexpr int kRouteBlockTokens = 64;  // tokens per block of the route kernels, one histogram row each ...
constexpr int kWaveBlockTokens = 16;   // ... except the sixteen-lanes-per-token kernel (E > 32) on small batches: 4 wavefronts x 4 tokens
constexpr int kWaveSmallBatch = 2048;  // largest batch that uses the small blocks (more blocks would swamp the plan kernel's sum)
inline __host__ __device__ int route_block_tokens(int E, int T) {
  return (E <= 32 || T > kWaveSmallBatch) ? kRouteBlockTokens : kWaveBlockTokens;
}

// MFMA path tile shape: 256 rows (token-expert pairs) x 128 neurons (gate+up = 256 weight rows)
// for GEMM-1, 256 rows x 256 output columns for GEMM-2, K stage 32.
constexpr int kMfmaBM = 256;
constexpr int kMfmaNeur = 128;
constexpr int kMfmaBN2 = 256;
constexpr int kBK = 32;                     // K values per pipeline stage
constexpr int kChunksPerRow = kBK / 8;      // 16-byte chunks in one tile row
constexpr int kStageBytes = 256 * kBK * 2;  // one operand tile of one stage (bf16): 16 KiB

// generic path tile shape
constexpr int kGenBM = 64;
constexpr int kGenBN = 64;

struct Item1 {  // one tile of GEMM-1: rows [row0, row0+nrows) x neurons tile jt of partition p
  int32_t row0, nrows, e, p, jt;
  int32_t nfill;  // rows of the whole row tile (>= nrows): rows [nrows, nfill) keep nothing of p and get zeros
  int32_t half;   // 0: the whole neuron tile; 1 / 2: its first / second 64 neurons (MFMA path, at most 128 rows)
  int32_t pad;
};
struct Item2 {  // one tile of GEMM-2: rows x output column tile jd, summed over partitions in kmask
  int32_t row0, nrows, e, jd, kmask;
  int32_t ks_lo, ks_n;  // K stages [ks_lo, ks_lo + ks_n) of every kept partition (the whole partition unless K is split)
  int32_t split;        // 0: the item writes its rows of Yp; n > 0: it writes partial-output tile n-1 of the pool
};

// Everything the device code needs to know about the layer and the workspace.
struct Layout {
  // layer
  int32_t D, F, E, K, P, Fp;
  int32_t lo, hi, E_res;      // resident window
  int32_t n_shared, F_shT;    // shared experts fused into one pseudo-expert of F_shT neurons (id E_res)
  int32_t renorm, dtype, mfma, router_mfma;
  int32_t y_f32;  // 1: y is float even though the layer's tensors are bf16
  int32_t yp_half;  // MFMA path: GEMM-2 stores its per-pair partial outputs (Yp, pool tiles) in half precision (times kYpHalfScale)
  int32_t h_shift;  // MFMA path: the intermediate activation is stored times 2^h_shift (folded into the packed W3)
  int32_t g2_rows_inner;  // GEMM-2 item order: 1 = (expert, column tile, row tile), 0 = (expert, row tile, column tile)
  int32_t tall_tiles;     // MFMA path: a GEMM item of a full row tile may also take the expert's last row tile if that has at most
                          // kTallExtra rows: 0 never, 1 where the plan's estimate says it pays (GEMM-1; always in GEMM-2), 2 wherever possible
  int32_t split_items;  // kSplitItems if GEMM-2 may split K (MFMA path), else 0
  int32_t max_tokens;
  // plan geometry
  int32_t BM;                 // row tile height
  int32_t NT1, NT1_sh;        // neuron tiles per partition (routed / shared)
  int32_t ND2;                // output column tiles of GEMM-2
  int32_t nsub, nbins;        // sort bins: E_res * nsub
  int32_t sh_rows;            // rows of the shared region (multiple of BM), first in the row space: the context holds the
                              // capacity for max_tokens, the copy a call hands to its kernels the boundary for its T
  int32_t row_cap;            // total row capacity
  int32_t max_tiles, max_items1, max_items2;
  int32_t pool_tiles;         // partial-output tiles of the workspace (GEMM-2 K splits)
  // workspace byte offsets
  int64_t o_idx, o_w, o_keep, o_pair_row, o_bin_count, o_cursor, o_exp_nrows, o_exp_row0, o_counters;
  int64_t o_tile_bits, o_act_rank, o_items1, o_items2;
  int64_t o_row_token, o_row_bits, o_H, o_Hs, o_Yp, o_tau0, o_sel, o_logits, o_perm_check, o_pool, o_split_of, ws_bytes;
  // packed weights byte offsets
  int64_t p_w13, p_w2, p_sw13, p_sw2, p_scale, packed_bytes, router_bytes;  // p_scale: the W2 scale record (MFMA layout)
  int64_t w13_expert_bytes, w2_expert_bytes;  // strides between experts (mfma layout)
};

// A set-up step that HIP keeps per device (hipFuncSetAttribute, hipGetSymbolAddress): run once for
// every device, with that device current, from whichever host thread gets there first.
constexpr int kMaxDevices = 64;
struct PerDeviceOnce {
  std::mutex mu;
  bool done[kMaxDevices] = {};
  template <class F>
  hipError_t run(F&& f) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return f();  // beyond the table: every time
    std::lock_guard<std::mutex> g(mu);
    if (done[dev]) return hipSuccess;
    e = f();
    if (e == hipSuccess) done[dev] = true;
    return e;
  }
};

constexpr int kNumKernels = 7;  // router (if any), route, plan, scatter, gemm1, gemm2, combine

struct Profile {
  int level = 0;       // 0 off, 1 GEMM-1 only, 2 every kernel
  int max_calls = 0;
  int calls = 0;
  hipEvent_t* ev = nullptr;  // level 1: 2 per call; level 2: kNumKernels + 1 per call
};

struct Ctx {
  dsmoe_config cfg;
  Layout L;
  int last_hip;
  int last_sh_rows;  // rows the last call reserved for the shared experts (for dsmoe_plan_layout)
  Profile prof;
};

// upper bounds of the plan sizes for a call with T tokens (the exact sizes only exist on the device)
inline int routed_tiles_bound(const Layout& L, int T) { return (int)(((int64_t)T * L.K) / L.BM) + L.E_res; }
inline int shared_tiles(const Layout& L, int T) { return L.n_shared > 0 ? (T + L.BM - 1) / L.BM : 0; }
inline int items1_whole_bound(const Layout& L, int T) {
  return routed_tiles_bound(L, T) * L.P * L.NT1 + shared_tiles(L, T) * L.NT1_sh;
}
// A last round of items may be cut into halves only in the weight-streaming regime: at most half a
// tile of rows per expert on average.
__host__ __device__ inline bool may_halve_items1(const Layout& L, int T) {
  return L.split_items > 0 && (int64_t)T * L.K <= (int64_t)L.E_res * (L.BM / 2);
}
inline int items1_bound(const Layout& L, int T) {
  return items1_whole_bound(L, T) + (may_halve_items1(L, T) ? L.split_items / 2 : 0);
}
inline int items2_bound(const Layout& L, int T) {
  const int whole = (routed_tiles_bound(L, T) + shared_tiles(L, T)) * L.ND2;
  return whole + L.pool_tiles;  // every extra K range of a split item is one more item
}

// launchers (each returns hipError_t of the launch)
hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t s);
hipError_t launch_route(const Layout& L, const float* logits, int T, const float* tau, int32_t* idx, float* w,
                        uint8_t* keep, int32_t* bin_count, int32_t* group_count, hipStream_t s, bool whole_router_scores = false);
hipError_t launch_plan(const Layout& L, int T, char* ws, hipStream_t s);
hipError_t launch_scatter(const Layout& L, int T, char* ws, hipStream_t s);
hipError_t launch_combine(const Layout& L, int T, const char* packed, char* ws, void* y, hipStream_t s);
// epi: what GEMM-1 stores per (row, neuron): 0 = Swish(gate)*up (the layer), 1..4 = the profiling
// metrics Swish(gate), |Swish(gate)|, Swish(gate)*up, |Swish(gate)*up|
hipError_t launch_gemm1_generic(const Layout& L, int T, const char* packed, const void* x, char* ws, int epi, hipStream_t s);
hipError_t launch_gemm2_generic(const Layout& L, int T, const char* packed, char* ws, hipStream_t s);
hipError_t launch_gemm1_mfma(const Layout& L, int T, const char* packed, const void* x, char* ws, int epi, hipStream_t s);
hipError_t launch_select_thresholds(const Layout& L, int T, const float* tau_max, int group_size, int row_cap, char* ws,
                                    float* tau, int32_t* pair_count, hipStream_t s);
hipError_t launch_router_pack(const Layout& L, const void* wg, char* out, hipStream_t s);
hipError_t launch_router(const Layout& L, int T, const char* router_packed, const void* x, float* logits, hipStream_t s);
hipError_t launch_transform_complete(const Layout& L, const void* wg, const void* w1, const void* w3, const void* w2,
                                     const int32_t* perm, void* wg_out, void* w1_out, void* w3_out, void* w2_out,
                                     hipStream_t s);
hipError_t launch_drop_rate_thresholds(const Layout& L, int T, double rate, const int32_t* offset_bins, char* ws, float* tau,
                                       int32_t* stats, hipStream_t s);
hipError_t launch_colsum(const Layout& L, const char* ws, int metric, float* importance, hipStream_t s);
hipError_t launch_perm_from_importance(const Layout& L, const float* importance, int32_t* perm, hipStream_t s);
hipError_t launch_gemm2_mfma(const Layout& L, int T, const char* packed, char* ws, hipStream_t s);
hipError_t launch_pack(const Layout& L, const void* w1, const void* w3, const void* w2, const void* sw1, const void* sw3,
                       const void* sw2, const int32_t* perm, char* packed, int n_shared, int F_sh, hipStream_t s);
hipError_t launch_perm_check(const Layout& L, const int32_t* perm, int32_t* scratch, hipStream_t s);

// ---- device helpers ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {  // round to nearest, ties to even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float silu_f32(float a) { return a / (1.0f + expf(-a)); }       // Swish, beta = 1
__device__ __forceinline__ float silu_fast(float a) { return a * __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }
// value GEMM-1 stores for gate g and up u (see launch_gemm1_*): Eq. 4's inner term, or one of the
// four importance metrics of Sec. 4.2 b
template <bool FAST>
__device__ __forceinline__ float epi_value(int epi, float g, float u) {
  const float sg = FAST ? silu_fast(g) : silu_f32(g);
  switch (epi) {
    case 1: return sg;
    case 2: return fabsf(sg);
    case 4: return fabsf(sg * u);
    default: return sg * u;  // 0 (layer) and 3
  }
}

// All-reductions inside a row of sixteen lanes: four data-parallel steps (mirror, half mirror, two
// quad permutations) leave the result in every lane of the row, with no LDS or scalar round trip.
constexpr int kRowMirror = 0x140, kRowHalfMirror = 0x141, kQuadSwap2 = 0x4E, kQuadSwap1 = 0xB1;
template <int CTRL>
__device__ __forceinline__ int dpp_all(int v) {
  return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ float row_max(float v) {
  v = fmaxf(v, __int_as_float(dpp_all<kRowMirror>(__float_as_int(v))));
  v = fmaxf(v, __int_as_float(dpp_all<kRowHalfMirror>(__float_as_int(v))));
  v = fmaxf(v, __int_as_float(dpp_all<kQuadSwap2>(__float_as_int(v))));
  v = fmaxf(v, __int_as_float(dpp_all<kQuadSwap1>(__float_as_int(v))));
  return v;
}
__device__ __forceinline__ float row_sum(float v) {  // every step adds two partners' values: the same bits in every lane
  v += __int_as_float(dpp_all<kRowMirror>(__float_as_int(v)));
  v += __int_as_float(dpp_all<kRowHalfMirror>(__float_as_int(v)));
  v += __int_as_float(dpp_all<kQuadSwap2>(__float_as_int(v)));
  v += __int_as_float(dpp_all<kQuadSwap1>(__float_as_int(v)));
  return v;
}

// Position of the 16-byte chunk `chunk` (0..3) of row `row` inside a [rows][32] bf16 LDS tile
// (64-byte rows).  The chunks of a row are XOR-rotated by bits 2..3 of the row so that an MFMA
// operand read (consecutive rows, same logical chunk) touches every LDS bank once per 16 lanes.
// XOR is its own inverse: the same function maps physical to logical positions.
__device__ __host__ __forceinline__ int swz_chunk(int row, int chunk) { return chunk ^ ((row >> 2) & 3); }

}  // namespace dsmoe
